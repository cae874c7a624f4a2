"""HIP path vs oracle, element by element, through the C ABI (needs an MI355X).

Bars: attention within 2e-2 absolute (bf16 I/O, fp32 softmax against the fp64
oracle); scores within 1e-5 relative; retained position sets and the K/V row
behind every retained position bit-exact.
"""
import os

import numpy as np
import pytest

import oracle
import paper_2504_15364_amd as kd
from helpers import (ATTN_ATOL, SCORE_ATOL, SCORE_RTOL, bf16_out_to_f32, blocks, rows_by_position, to_dev)
from synth import apply_rope, bf16_bits_to_f32, block_of, f32_to_bf16_bits, get_config, make_layer, rope_tables

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def make_pair(w, N, B, batch=1, **kw):
    cfg = kd.KeyDiffConfig(batch, w.n_q_heads, w.n_kv_heads, w.head_dim, N, B, **kw)
    okw = {k: v for k, v in kw.items() if k != "layout"}
    return kd.KeyDiffCache(cfg), oracle.OracleCache(batch, w.n_q_heads, w.n_kv_heads, w.head_dim, N, B, **okw)


def check_state(cache, oc, where):
    pos, K, V = rows_by_position(cache)
    assert cache.len == oc.len, where
    assert np.array_equal(pos, oc.positions()), f"retained positions differ {where}"
    assert np.array_equal(K, oc.keys()), f"K rows differ {where}"
    assert np.array_equal(V, oc.values()), f"V rows differ {where}"
    if cache.cfg.layout == kd.LAYOUT_ORDERED:
        raw = cache.positions().cpu().numpy()
        assert np.all(np.diff(raw, axis=-1) > 0), f"ORDERED layout not ascending {where}"


def run_prompt(w, data, N, B, T=None, check_scores=True, **kw):
    cache, oc = make_pair(w, N, B, **kw)
    worst = 0.0
    for t, Bt, q, k, v in blocks(data, B, T):
        n = cache.len + Bt
        pos_before = np.concatenate(
            [cache.positions().cpu().numpy(), np.broadcast_to(np.arange(t, t + Bt, dtype=np.int32), (1, w.n_kv_heads, Bt))],
            axis=-1)
        sc = torch.empty((1, w.n_kv_heads, n), dtype=torch.float32, device="cuda") if check_scores else None
        out = cache.prefill_block(to_dev(q), to_dev(k), to_dev(v), t, scores_out=sc)
        ref, osc, ev = oc.prefill_block(q, k, v, t, want_scores=True)
        err = float(np.abs(bf16_out_to_f32(out) - ref).max())
        worst = max(worst, err)
        assert err <= ATTN_ATOL, f"attention error {err} in block at token {t}"
        if check_scores and ev > 0:
            # the oracle lists rows by ascending position; map the HIP row order onto it
            order = np.argsort(pos_before, axis=-1, kind="stable")
            got = np.take_along_axis(sc.cpu().numpy(), order, axis=-1)
            assert np.allclose(got, osc, rtol=SCORE_RTOL, atol=SCORE_ATOL), f"scores differ at token {t}"
        check_state(cache, oc, f"after the block at token {t}")
    assert cache.status() == 0
    cache.close()
    return worst


@pytest.mark.parametrize("layout", [kd.LAYOUT_ORDERED, kd.LAYOUT_FILL])
def test_toy_config_whole_prompt(layout):
    w = get_config("toy")
    data = make_layer(w, seed=1)
    run_prompt(w, data, w.budget_N, w.block_B, layout=layout)


@pytest.mark.parametrize("layout", [kd.LAYOUT_ORDERED, kd.LAYOUT_FILL])
@pytest.mark.parametrize("hq,hkv,d,N,B,T", [
    (6, 2, 128, 200, 48, 500),     # G = 3, tiles ragged in keys and rows, ragged last block
    (8, 2, 64, 130, 100, 650),     # first eviction evicts fewer rows than the block holds
    (14, 2, 128, 320, 64, 448),    # G = 7 (Qwen-style group)
    (4, 4, 128, 70, 7, 120),       # tiny blocks, budget below one key tile
])
def test_ragged_shapes(layout, hq, hkv, d, N, B, T):
    w = get_config("llama32_3b").small(n_q_heads=hq, n_kv_heads=hkv, head_dim=d, prompt_T=T)
    data = make_layer(w, seed=100 + hq + N)
    run_prompt(w, data, N, B, layout=layout)


def test_two_row_tiles_per_head_and_split_merge():
    # G * B = 512 rows per KV head: two 256-row workgroup tiles per head and several key splits
    w = get_config("llama31_8b").small(n_q_heads=8, n_kv_heads=2, prompt_T=1536)
    data = make_layer(w, seed=5)
    run_prompt(w, data, 768, 128, layout=kd.LAYOUT_FILL)


@pytest.mark.parametrize("layout", [kd.LAYOUT_ORDERED, kd.LAYOUT_FILL])
@pytest.mark.parametrize("shape", ["toy", "ragged"])
def test_unit_key_anchor(layout, shape):
    # Eq. 7 literally: the anchor is the mean of the unit keys (anchor_mode = 1); the running sum of
    # unit keys goes through the same append / evict updates as the raw-key sum
    if shape == "toy":
        w = get_config("toy")
        N, B = w.budget_N, w.block_B
    else:
        w = get_config("llama32_3b").small(n_q_heads=6, n_kv_heads=2, head_dim=128, prompt_T=500)
        N, B = 200, 48
    data = make_layer(w, seed=31)
    run_prompt(w, data, N, B, layout=layout, anchor_mode=kd.ANCHOR_MEAN_UNIT_KEY)


@pytest.mark.parametrize("layout", [kd.LAYOUT_ORDERED, kd.LAYOUT_FILL])
@pytest.mark.parametrize("frac", [0.1, 0.2])
def test_sliding_window_is_exempt_from_eviction(layout, frac):
    # Method, "KeyDiff with Sliding Window": the W most recent tokens always stay, KeyDiff picks
    # the rest of the budget (the paper uses 10 % and 20 % of the budget)
    w = get_config("toy")
    N, B = w.budget_N, w.block_B
    W = int(frac * N)
    data = make_layer(w, seed=32)
    cache, oc = make_pair(w, N, B, layout=layout, window_W=W)
    for t, Bt, q, k, v in blocks(data, B):
        out = cache.prefill_block(to_dev(q), to_dev(k), to_dev(v), t)
        ref, _, ev = oc.prefill_block(q, k, v, t)
        assert np.abs(bf16_out_to_f32(out) - ref).max() <= ATTN_ATOL
        check_state(cache, oc, f"window {W}, block at token {t}")
        if ev > 0:
            kept = np.sort(cache.positions().cpu().numpy(), axis=-1)
            assert np.all(kept[..., -W:] == np.arange(t + Bt - W, t + Bt)), "a window token was evicted"
    assert cache.status() == 0
    cache.close()


def test_window_with_unit_key_anchor_large_group():
    w = get_config("llama32_3b").small(n_q_heads=14, n_kv_heads=2, head_dim=128, prompt_T=448)
    data = make_layer(w, seed=33)
    run_prompt(w, data, 320, 64, layout=kd.LAYOUT_FILL, anchor_mode=kd.ANCHOR_MEAN_UNIT_KEY, window_W=64)


def test_budget_not_reached_only_appends():
    w = get_config("toy").small(prompt_T=96)
    data = make_layer(w, seed=2)
    cache, oc = make_pair(w, 128, 32)
    for t, Bt, q, k, v in blocks(data, 32):
        out = cache.prefill_block(to_dev(q), to_dev(k), to_dev(v), t)
        ref, _, ev = oc.prefill_block(q, k, v, t)
        assert ev == 0 and np.abs(bf16_out_to_f32(out) - ref).max() <= ATTN_ATOL
    assert cache.len == 96
    check_state(cache, oc, "no eviction")


def test_prefill_of_a_batch_of_sequences():
    # several independent sequences in one call: per-sequence caches, positions and retained sets
    w = get_config("llama32_3b").small(n_q_heads=6, n_kv_heads=2, head_dim=128, prompt_T=480, batch=3)
    N, B = 200, 48
    seqs = [make_layer(w, seed=61, seq=s_) for s_ in range(w.batch)]
    cache, oc = make_pair(w, N, B, batch=w.batch, layout=kd.LAYOUT_FILL)
    for t in range(0, w.prompt_T, B):
        q, k, v = (np.stack([block_of(s_[x], t, B) for s_ in seqs]) for x in ("q", "k", "v"))
        out = cache.prefill_block(to_dev(q), to_dev(k), to_dev(v), t)
        ref, _, _ = oc.prefill_block(q, k, v, t)
        assert np.abs(bf16_out_to_f32(out) - ref).max() <= ATTN_ATOL, t
        check_state(cache, oc, f"batch of {w.batch}, token {t}")
    assert cache.status() == 0


def test_more_heads_than_compute_units():
    # batch x KV heads x row tiles beyond the 256 compute units: one key split, workgroups in rounds
    w = get_config("toy").small(n_q_heads=2, n_kv_heads=2, head_dim=64, prompt_T=96, batch=150)
    N, B = 48, 16
    seqs = [make_layer(w, seed=62, seq=s_) for s_ in range(w.batch)]
    cache, oc = make_pair(w, N, B, batch=w.batch, layout=kd.LAYOUT_FILL)
    for t in range(0, w.prompt_T, B):
        q, k, v = (np.stack([block_of(s_[x], t, B) for s_ in seqs]) for x in ("q", "k", "v"))
        out = cache.prefill_block(to_dev(q), to_dev(k), to_dev(v), t)
        ref, _, _ = oc.prefill_block(q, k, v, t)
        assert np.abs(bf16_out_to_f32(out) - ref).max() <= ATTN_ATOL, t
    check_state(cache, oc, "300 heads")
    assert cache.status() == 0


@pytest.mark.parametrize("layout", [kd.LAYOUT_ORDERED, kd.LAYOUT_FILL])
def test_decode_steps_batch(layout):
    # B = 1 is the generation phase: several independent sequences, one eviction per step
    w = get_config("decode_8b").small(n_q_heads=8, n_kv_heads=2, prompt_T=200, batch=3)
    N = 150
    seqs = [make_layer(w, seed=9, seq=s) for s in range(w.batch)]
    cache, oc = make_pair(w, N, 1, batch=w.batch, layout=layout)
    for t in range(w.prompt_T):
        q, k, v = (np.stack([s[x][t][:, None, :] for s in seqs]) for x in ("q", "k", "v"))
        out = cache.decode_step(to_dev(q), to_dev(k), to_dev(v), t)
        ref, _, ev = oc.decode_step(q, k, v, t)
        assert np.abs(bf16_out_to_f32(out) - ref).max() <= ATTN_ATOL, t
        assert ev == (1 if t >= N else 0)
        if t % 25 == 0 or t > 190:
            check_state(cache, oc, f"decode step {t}")
    check_state(cache, oc, "end of decode")
    assert cache.status() == 0


@pytest.mark.parametrize("kw", [dict(anchor_mode=kd.ANCHOR_MEAN_UNIT_KEY), dict(window_W=12),
                                dict(anchor_mode=kd.ANCHOR_MEAN_UNIT_KEY, window_W=30)])
def test_decode_steps_unit_anchor_and_window(kw):
    # one eviction per step takes the arg-max path of the selection: cover its unit-key sum update and
    # the window exemption (also the step whose own token is the one evicted)
    w = get_config("decode_8b").small(n_q_heads=8, n_kv_heads=2, prompt_T=160, batch=2)
    N = 96
    seqs = [make_layer(w, seed=19, seq=s) for s in range(w.batch)]
    cache, oc = make_pair(w, N, 1, batch=w.batch, layout=kd.LAYOUT_FILL, **kw)
    for t in range(w.prompt_T):
        q, k, v = (np.stack([s[x][t][:, None, :] for s in seqs]) for x in ("q", "k", "v"))
        out = cache.decode_step(to_dev(q), to_dev(k), to_dev(v), t)
        ref, _, ev = oc.decode_step(q, k, v, t)
        assert np.abs(bf16_out_to_f32(out) - ref).max() <= ATTN_ATOL, t
        if t % 16 == 0 or t > 150:
            check_state(cache, oc, f"decode step {t}")
    check_state(cache, oc, "end of decode")
    assert cache.status() == 0


def test_decode_ties_are_decided_by_position_not_by_row():
    # generation phase, FILL layout: the attention launch hands the selection the arg-max by (score, row) of
    # every workgroup; where several rows share the largest score the lower POSITION must stay, and after a
    # few hole fills positions are no longer in row order.  Half of the tokens repeat one key exactly.
    w = get_config("decode_8b").small(n_q_heads=8, n_kv_heads=2, prompt_T=260, batch=2)
    N = 160
    seqs = [make_layer(w, seed=29, seq=s) for s in range(w.batch)]
    for s_ in seqs:
        s_["k"][1::2] = s_["k"][1]          # every odd token carries the key of token 1
    cache, oc = make_pair(w, N, 1, batch=w.batch, layout=kd.LAYOUT_FILL)
    for t in range(w.prompt_T):
        q, k, v = (np.stack([s_[x][t][:, None, :] for s_ in seqs]) for x in ("q", "k", "v"))
        out = cache.decode_step(to_dev(q), to_dev(k), to_dev(v), t)
        ref, _, ev = oc.decode_step(q, k, v, t)
        assert np.abs(bf16_out_to_f32(out) - ref).max() <= ATTN_ATOL, t
        if t >= N:
            check_state(cache, oc, f"decode step {t}")
    assert cache.status() == 0


@pytest.mark.parametrize("layout", [kd.LAYOUT_ORDERED, kd.LAYOUT_FILL])
def test_ties_keep_the_lower_position(layout):
    # identical keys: every score is equal, so each step must evict the highest positions
    hq, hkv, d, N, B = 2, 1, 64, 96, 32
    w = get_config("toy").small(n_q_heads=hq, n_kv_heads=hkv, head_dim=d, prompt_T=256)
    data = make_layer(w, seed=3)
    same = f32_to_bf16_bits(np.tile(np.linspace(-1, 2, d, dtype=np.float32), (256, hkv, 1)))
    data = dict(data, k=same)
    cache, oc = make_pair(w, N, B, layout=layout)
    for t, Bt, q, k, v in blocks(data, B):
        cache.prefill_block(to_dev(q), to_dev(k), to_dev(v), t)
        oc.prefill_block(q, k, v, t)
        check_state(cache, oc, f"ties, token {t}")
    assert np.array_equal(np.sort(cache.positions().cpu().numpy())[0, 0], np.arange(N))


def test_thousands_of_identical_keys_take_the_radix_path():
    # every score equal: the threshold bin holds all rows (more than the LDS ranking takes), so the
    # selection falls back to the radix select on (score bits, position); the survivors must be the
    # N lowest positions
    hq, hkv, d, N, B = 2, 1, 64, 2560, 512
    T = N + 2 * B
    w = get_config("toy").small(n_q_heads=hq, n_kv_heads=hkv, head_dim=d, prompt_T=T)
    data = make_layer(w, seed=13)
    same = f32_to_bf16_bits(np.tile(np.linspace(0.5, 1.5, d, dtype=np.float32), (T, hkv, 1)))
    data = dict(data, k=same)
    cache, oc = make_pair(w, N, B, layout=kd.LAYOUT_FILL)
    for t, Bt, q, k, v in blocks(data, B):
        cache.prefill_block(to_dev(q), to_dev(k), to_dev(v), t)
        oc.prefill_block(None, k, v, t)
    check_state(cache, oc, "identical keys")
    assert np.array_equal(np.sort(cache.positions().cpu().numpy())[0, 0], np.arange(N))
    assert cache.status() == 0


@pytest.mark.parametrize("layout", [kd.LAYOUT_ORDERED, kd.LAYOUT_FILL])
def test_block_larger_than_the_budget(layout):
    # the very first block overflows the budget: rows are evicted before any was ever kept
    w = get_config("toy").small(n_q_heads=4, n_kv_heads=2, head_dim=64, prompt_T=192)
    data = make_layer(w, seed=14)
    run_prompt(w, data, 16, 64, layout=layout)


def _random_configs(count, seed):
    """Seeded draws of small shapes: group sizes 1-7, both head sizes, block sizes from 1 to a few tiles, budgets
    from below one key tile to a dozen, ragged prompts, both layouts, both anchors, an occasional window."""
    rng = np.random.default_rng(seed)
    out = []
    for i in range(count):
        hkv = int(rng.integers(1, 4))
        G = int(rng.choice([1, 2, 3, 4, 7]))
        d = int(rng.choice([64, 128]))
        B = int(rng.choice([1, 3, 16, 40, 64, 100, 128, 160]))
        N = int(rng.integers(max(B // 2, 8), 700))
        steps = int(rng.integers(3, 7)) if B > 1 else int(rng.integers(20, 40))
        T = N + steps * B + int(rng.integers(0, B))
        layout = int(rng.choice([kd.LAYOUT_FILL, kd.LAYOUT_ORDERED]))
        anchor = int(rng.choice([kd.ANCHOR_MEAN_KEY, kd.ANCHOR_MEAN_UNIT_KEY]))
        window = int(rng.integers(1, max(2, N // 4))) if rng.random() < 0.25 else 0
        out.append(pytest.param(hkv * G, hkv, d, N, B, T, layout, anchor, window, 9000 + i,
                                id=f"{i}-hq{hkv * G}-hkv{hkv}-d{d}-N{N}-B{B}-T{T}-l{layout}-a{anchor}-w{window}"))
    return out


# (KEYDIFF_FUZZ multiplies the number of drawn configurations, for an occasional longer run)
FUZZ = max(1, int(os.environ.get("KEYDIFF_FUZZ", "1")))


@pytest.mark.parametrize("hq,hkv,d,N,B,T,layout,anchor,window,seed", _random_configs(16 * FUZZ, 20250415))
def test_seeded_random_small_configs(hq, hkv, d, N, B, T, layout, anchor, window, seed):
    w = get_config("llama32_3b").small(n_q_heads=hq, n_kv_heads=hkv, head_dim=d, prompt_T=T)
    data = make_layer(w, seed=seed)
    run_prompt(w, data, N, B, layout=layout, anchor_mode=anchor, window_W=window)


@pytest.mark.parametrize("d,N,B,T", [(128, 640, 600, 1900), (64, 768, 700, 2200)], ids=["d128", "d64"])
def test_blocks_longer_than_the_rows_requested_up_front(d, N, B, T):
    # the attention kernel requests the first 256 (d = 128) or 512 (d = 64) rows of a block ahead of its
    # tile copies for the key sum; longer blocks take further batches, and a ragged last one
    w = get_config("toy").small(n_q_heads=2, n_kv_heads=1, head_dim=d, prompt_T=T)
    data = make_layer(w, seed=16 + d)
    run_prompt(w, data, N, B, layout=kd.LAYOUT_FILL)


def test_single_tokens_from_an_empty_cache():
    # B = 1 from the first token on: one-key attention, then one eviction per step once full
    w = get_config("toy").small(n_q_heads=4, n_kv_heads=2, head_dim=128, prompt_T=40)
    data = make_layer(w, seed=15)
    run_prompt(w, data, 24, 1, layout=kd.LAYOUT_FILL)


def test_largest_capacity():
    # budget_N + block_B at the limit of the library (32768 rows): the large selection instantiation,
    # lists in device memory, 512 key tiles.  One head pair keeps the oracle fast; the cache is brought
    # to the budget by a load, then two block steps run, the first with attention checked.
    hq, hkv, d, B = 2, 1, 128, 256
    N = 32768 - B
    w = get_config("llama31_8b").small(n_q_heads=hq, n_kv_heads=hkv, head_dim=d, prompt_T=N + 2 * B)
    data = make_layer(w, seed=16)
    cache, oc = make_pair(w, N, B, layout=kd.LAYOUT_FILL)
    K0 = data["k"][:N].transpose(1, 0, 2)[None].copy()
    V0 = data["v"][:N].transpose(1, 0, 2)[None].copy()
    P0 = np.broadcast_to(np.arange(N, dtype=np.int32), (1, hkv, N)).copy()
    cache.load(to_dev(K0), to_dev(V0), torch.from_numpy(P0).cuda())
    oc.load(K0, V0, P0)
    for i, (t, Bt, q, k, v) in enumerate(b for b in blocks(data, B) if b[0] >= N):
        out = cache.prefill_block(to_dev(q), to_dev(k), to_dev(v), t)
        ref, _, ev = oc.prefill_block(q if i == 0 else None, k, v, t)
        assert ev == B
        if i == 0:
            assert np.abs(bf16_out_to_f32(out) - ref).max() <= ATTN_ATOL
        check_state(cache, oc, f"largest capacity, token {t}")
    assert cache.status() == 0
    cache.close()



# ---- deferred eviction: the selection of one layer rides in the attention launch of the next ----
def run_layers_deferred(w, N, B, nlayers, seeds, check_every, expect_ride, datas=None, **kw):
    """Layers run in turn on every block, each carrying the pending eviction of the one before it
    (the first carries the last one's from the previous block).  Attention is checked on every
    call; the cache states every `check_every` blocks (reading a state finishes its pending
    eviction in a launch of its own) and at the end."""
    layers = [make_pair(w, N, B, **kw) for _ in range(nlayers)]
    datas = datas or [make_layer(w, seed=s) for s in seeds]
    for c, _ in layers:
        c.profile_enable(True)
    evicting = 0
    for bi, steps in enumerate(zip(*(blocks(d, B) for d in datas))):
        for li, (t, Bt, q, k, v) in enumerate(steps):
            cache, oc = layers[li]
            carry = layers[li - 1][0] if nlayers > 1 else None
            out = cache.prefill_block_deferred(to_dev(q), to_dev(k), to_dev(v), t, carry=carry)
            ref, _, ev = oc.prefill_block(q, k, v, t)
            err = float(np.abs(bf16_out_to_f32(out) - ref).max())
            assert err <= ATTN_ATOL, f"attention error {err}, layer {li}, block at token {t}"
            evicting += int(ev > 0 and li == 0)
        if check_every and bi % check_every == check_every - 1:
            for li, (cache, oc) in enumerate(layers):
                check_state(cache, oc, f"layer {li} after block {bi}")
    for li, (cache, oc) in enumerate(layers):
        check_state(cache, oc, f"layer {li} at the end")
        assert cache.status() == 0
    counts = [c.profile_read() for c, _ in layers]
    for c, _ in layers:
        c.close()
    if expect_ride is not None:
        alone = sum(cnt["select_alone"][1] for cnt in counts)   # evictions finished in a launch of their own
        if expect_ride:
            # only what the state checks and the end of the run forced out
            forced = nlayers * ((len(list(blocks(datas[0], B))) // check_every if check_every else 0) + 1)
            assert 0 <= alone <= forced, (alone, forced)
            assert evicting * nlayers - alone > 0, "no eviction rode along"
        else:
            assert alone >= evicting * nlayers - nlayers, alone


def test_deferred_eviction_rides_the_next_layers_attention():
    # G * B = 512 rows per KV head: 8-wave workgroups, several key splits, the carrying kernel
    w = get_config("llama31_8b").small(n_q_heads=8, n_kv_heads=2, prompt_T=1536)
    run_layers_deferred(w, 768, 128, 3, seeds=(41, 42, 43), check_every=0, expect_ride=True, layout=kd.LAYOUT_FILL)


@pytest.mark.parametrize("N,B", [(448, 64), (1536, 64)], ids=["ranked-in-lds", "radix-select"])
@pytest.mark.parametrize("layout", [kd.LAYOUT_FILL, kd.LAYOUT_ORDERED], ids=["fill", "ordered"])
def test_deferred_eviction_of_nearly_identical_keys(N, B, layout):
    # Keys that differ from one common vector in a single component by one bf16 step have scores
    # 1e-8 .. 1e-6 apart, many of them equal once rounded to float (the position then decides): the
    # threshold bin of the selection holds every row.  With 512 rows they fit its candidate table, with
    # 1600 they take the radix select; the evictions ride in the next layer's attention launch.
    w = get_config("llama31_8b").small(n_q_heads=8, n_kv_heads=2, prompt_T=N + 4 * B)
    rng = np.random.default_rng(N)
    datas = []
    for seed in (71, 72):
        data = make_layer(w, seed=seed)
        base = np.linspace(-1.0, 2.0, w.head_dim, dtype=np.float32)
        k = np.tile(base, (w.prompt_T, w.n_kv_heads, 1))
        cols = rng.integers(0, w.head_dim, size=(w.prompt_T, w.n_kv_heads))
        bits = f32_to_bf16_bits(k)
        step = rng.integers(-1, 2, size=(w.prompt_T, w.n_kv_heads)).astype(np.int32)   # -1, 0 or +1 bf16 steps
        tt, hh = np.meshgrid(np.arange(w.prompt_T), np.arange(w.n_kv_heads), indexing="ij")
        bits[tt, hh, cols] = (bits[tt, hh, cols].astype(np.int32) + step).astype(np.uint16)
        datas.append(dict(data, k=bits))
    run_layers_deferred(w, N, B, 2, seeds=None, check_every=1, expect_ride=None, datas=datas, layout=layout)
    run_layers_deferred(w, N, B, 2, seeds=None, check_every=0, expect_ride=True, datas=datas, layout=layout)


def test_deferred_eviction_with_states_read_in_between():
    # reading a cache finishes its eviction alone: riding and stand-alone finishes interleave
    w = get_config("llama31_8b").small(n_q_heads=8, n_kv_heads=2, prompt_T=1280)
    run_layers_deferred(w, 640, 128, 2, seeds=(44, 45), check_every=3, expect_ride=True, layout=kd.LAYOUT_FILL,
                        anchor_mode=kd.ANCHOR_MEAN_UNIT_KEY, window_W=64)


def test_deferred_eviction_where_nothing_can_ride():
    # with a single wave's worth of query rows per head the attention runs its alternating-waves mode,
    # which has no carrying variant: every eviction is finished in a launch of its own, in both
    # layouts, with the plain call's results
    w = get_config("llama32_3b").small(n_q_heads=4, n_kv_heads=2, head_dim=128, prompt_T=240)
    run_layers_deferred(w, 80, 8, 2, seeds=(46, 47), check_every=0, expect_ride=False, layout=kd.LAYOUT_FILL)
    run_layers_deferred(w, 80, 8, 2, seeds=(48, 49), check_every=0, expect_ride=False, layout=kd.LAYOUT_ORDERED)


def test_deferred_eviction_ordered_layout_rides_and_shifts_afterwards():
    # ORDERED layout: the selection rides in the next layer's attention launch, the stable row shift
    # follows in a launch of its own; rows stay in position order (check_state reads them by row)
    w = get_config("llama31_8b").small(n_q_heads=8, n_kv_heads=2, prompt_T=1536)
    run_layers_deferred(w, 768, 128, 3, seeds=(61, 62, 63), check_every=5, expect_ride=True, layout=kd.LAYOUT_ORDERED)
    # ragged last block, helper-wave variant, unit-key anchor and window
    w = get_config("llama32_3b").small(n_q_heads=6, n_kv_heads=2, head_dim=128, prompt_T=1100)
    run_layers_deferred(w, 384, 128, 2, seeds=(64, 65), check_every=0, expect_ride=True, layout=kd.LAYOUT_ORDERED,
                        anchor_mode=kd.ANCHOR_MEAN_UNIT_KEY, window_W=32)


def test_block_through_all_layers_in_one_call():
    # keydiff_prefill_block_layers: one call per block enqueues every layer, each carrying the one
    # before it; layer 0 carries the last layer's eviction of the previous block
    w = get_config("llama31_8b").small(n_q_heads=8, n_kv_heads=2, prompt_T=1408)
    N, B, nl = 640, 128, 4
    layers = [make_pair(w, N, B, layout=kd.LAYOUT_FILL) for _ in range(nl)]
    datas = [make_layer(w, seed=81 + l) for l in range(nl)]
    caches = [c for c, _ in layers]
    for c in caches:
        c.profile_enable(True)
    evicting = 0
    for steps in zip(*(blocks(d, B) for d in datas)):
        t = steps[0][0]
        outs = kd.prefill_block_layers(caches, [to_dev(s[2]) for s in steps], [to_dev(s[3]) for s in steps],
                                       [to_dev(s[4]) for s in steps], t)
        for (cache, oc), (_, Bt, q, k, v), out in zip(layers, steps, outs):
            ref, _, ev = oc.prefill_block(q, k, v, t)
            err = float(np.abs(bf16_out_to_f32(out) - ref).max())
            assert err <= ATTN_ATOL, f"attention error {err} in block at token {t}"
        evicting += int(ev > 0)
    alone = 0
    for li, (cache, oc) in enumerate(layers):
        check_state(cache, oc, f"layer {li} at the end")
        assert cache.status() == 0
        alone += cache.profile_read()["select_alone"][1]
        cache.close()
    assert evicting > 2 and alone == 1, (evicting, alone)   # only the last layer's last eviction ran alone
    # a single layer: nothing to carry, same results
    (cache, oc), data = make_pair(w, N, B, layout=kd.LAYOUT_ORDERED), make_layer(w, seed=90)
    for t, Bt, q, k, v in blocks(data, B):
        out, = kd.prefill_block_layers([cache], [to_dev(q)], [to_dev(k)], [to_dev(v)], t)
        ref, _, _ = oc.prefill_block(q, k, v, t)
        assert float(np.abs(bf16_out_to_f32(out) - ref).max()) <= ATTN_ATOL
    check_state(cache, oc, "single layer")
    # argument errors are reported before anything is enqueued
    with pytest.raises(kd.KeyDiffError):
        kd.prefill_block_layers([cache, cache], [to_dev(q)] * 2, [to_dev(k)] * 2, [to_dev(v)] * 2, 0)
    cache.close()


@pytest.mark.parametrize("check_every", [0, 3], ids=["undisturbed", "states-read-in-between"])
def test_ordered_layers_call_shifts_inside_later_attention_launches(check_every):
    # ORDERED layout through keydiff_prefill_block_layers with three layers or more: the selection of layer
    # l rides in the attention launch of layer l + 1 and the stable row shift by its destination map in
    # that of layer l + 2 (workgroups that own a range of 128-row chunks each).  Reading a cache's state
    # in between runs whatever is still pending for it in launches of its own.
    # (the last block is ragged: its launches have helper waves and take no shift along, so the shifts
    # still pending then are enqueued alone when the states are read)
    w = get_config("llama31_8b").small(n_q_heads=8, n_kv_heads=2, prompt_T=2000)
    N, B, nl = 1024, 128, 4      # 9 chunks per head: ranges of one and of two chunks
    layers = [make_pair(w, N, B, layout=kd.LAYOUT_ORDERED) for _ in range(nl)]
    datas = [make_layer(w, seed=131 + l) for l in range(nl)]
    caches = [c for c, _ in layers]
    hosted = 0
    for bi, steps in enumerate(zip(*(blocks(d, B) for d in datas))):
        t = steps[0][0]
        outs = kd.prefill_block_layers(caches, [to_dev(s[2]) for s in steps], [to_dev(s[3]) for s in steps],
                                       [to_dev(s[4]) for s in steps], t)
        hosted += sum(1 for c in caches if c.plan()[3] & 2)
        for (cache, oc), (_, Bt, q, k, v), out in zip(layers, steps, outs):
            ref, _, _ = oc.prefill_block(q, k, v, t)
            err = float(np.abs(bf16_out_to_f32(out) - ref).max())
            assert err <= ATTN_ATOL, f"attention error {err} in block at token {t}"
        if check_every and bi % check_every == check_every - 1:
            for li, (cache, oc) in enumerate(layers):
                check_state(cache, oc, f"layer {li} after block {bi}")
                assert np.all(np.diff(cache.positions().cpu().numpy(), axis=-1) > 0), "rows not in position order"
    for li, (cache, oc) in enumerate(layers):
        check_state(cache, oc, f"layer {li} at the end")
        assert np.all(np.diff(cache.positions().cpu().numpy(), axis=-1) > 0), "rows not in position order"
        assert cache.status() == 0
        cache.close()
    assert hosted >= 8, f"only {hosted} attention launches took a row shift along"


def _random_layer_configs(count, seed):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(count):
        hkv = int(rng.integers(1, 4))
        G = int(rng.choice([1, 2, 4, 7]))
        d = int(rng.choice([64, 128]))
        B = int(rng.choice([16, 64, 128, 256]))
        N = B * int(rng.integers(1, 6)) + int(rng.choice([0, 0, 24]))
        T = N + int(rng.integers(3, 6)) * B + int(rng.integers(0, B))
        nl = int(rng.integers(2, 6))
        layout = int(rng.choice([kd.LAYOUT_FILL, kd.LAYOUT_ORDERED]))
        every = int(rng.choice([0, 2]))
        out.append(pytest.param(hkv * G, hkv, d, N, B, T, nl, layout, every, 9500 + 10 * i,
                                id=f"{i}-hq{hkv * G}-hkv{hkv}-d{d}-N{N}-B{B}-T{T}-layers{nl}-l{layout}-every{every}"))
    return out


@pytest.mark.parametrize("hq,hkv,d,N,B,T,nl,layout,every,seed", _random_layer_configs(10 * FUZZ, 20250416))
def test_seeded_random_configs_through_the_layers_call(hq, hkv, d, N, B, T, nl, layout, every, seed):
    # keydiff_prefill_block_layers over drawn shapes: whichever way an eviction (and, ORDERED, its row shift) ends up
    # being run -- riding in a later launch, inside a merge launch, or alone when a state is read -- the
    # results are the oracle's
    w = get_config("llama32_3b").small(n_q_heads=hq, n_kv_heads=hkv, head_dim=d, prompt_T=T)
    layers = [make_pair(w, N, B, layout=layout) for _ in range(nl)]
    datas = [make_layer(w, seed=seed + l) for l in range(nl)]
    caches = [c for c, _ in layers]
    for bi, steps in enumerate(zip(*(blocks(dd, B) for dd in datas))):
        t = steps[0][0]
        outs = kd.prefill_block_layers(caches, [to_dev(s_[2]) for s_ in steps], [to_dev(s_[3]) for s_ in steps],
                                       [to_dev(s_[4]) for s_ in steps], t)
        for (cache, oc), (_, Bt, q, k, v), out in zip(layers, steps, outs):
            ref, _, _ = oc.prefill_block(q, k, v, t)
            err = float(np.abs(bf16_out_to_f32(out) - ref).max())
            assert err <= ATTN_ATOL, f"attention error {err} in block at token {t}"
        if every and bi % every == every - 1:
            for li, (cache, oc) in enumerate(layers):
                check_state(cache, oc, f"layer {li} after block {bi}")
    for li, (cache, oc) in enumerate(layers):
        check_state(cache, oc, f"layer {li} at the end")
        assert cache.status() == 0
        cache.close()


def test_deferred_eviction_rides_a_launch_with_helper_waves():
    # G * B = 384 rows per KV head: 8-wave workgroups of which the second row tile fills only half,
    # so the attention runs its helper-wave variant; passengers ride in that one too
    w = get_config("llama32_3b").small(n_q_heads=6, n_kv_heads=2, head_dim=128, prompt_T=1280)
    run_layers_deferred(w, 384, 128, 2, seeds=(51, 52), check_every=0, expect_ride=True, layout=kd.LAYOUT_FILL)


def test_deferred_eviction_head_dim_64():
    # the 64-wide instantiation of the carrying kernel (its LDS holds the selection's workspace with
    # little to spare at this head size)
    w = get_config("toy").small(n_q_heads=8, n_kv_heads=2, head_dim=64, prompt_T=1024)
    run_layers_deferred(w, 448, 64, 3, seeds=(71, 72, 73), check_every=4, expect_ride=True, layout=kd.LAYOUT_FILL)


def test_deferred_eviction_on_another_stream_is_finished_on_its_own():
    # a carrier on a different stream cannot take the eviction along: it is enqueued on the stream of
    # the call that deferred it, and both caches still end up right
    w = get_config("llama31_8b").small(n_q_heads=8, n_kv_heads=2, prompt_T=1024)
    N, B = 512, 128
    a, oa = make_pair(w, N, B, layout=kd.LAYOUT_FILL)
    b, ob = make_pair(w, N, B, layout=kd.LAYOUT_FILL)
    da, db = make_layer(w, seed=53), make_layer(w, seed=54)
    side = torch.cuda.Stream()
    for (t, Bt, qa, ka, va), (_, _, qb, kb, vb) in zip(blocks(da, B), blocks(db, B)):
        out_a = a.prefill_block_deferred(to_dev(qa), to_dev(ka), to_dev(va), t)
        ref_a, _, _ = oa.prefill_block(qa, ka, va, t)
        tq, tk, tv = to_dev(qb), to_dev(kb), to_dev(vb)
        torch.cuda.synchronize()            # the inputs are there before the side stream reads them
        with torch.cuda.stream(side):
            out_b = b.prefill_block_deferred(tq, tk, tv, t, carry=a, stream=side)
        ref_b, _, _ = ob.prefill_block(qb, kb, vb, t)
        torch.cuda.synchronize()
        assert np.abs(bf16_out_to_f32(out_a) - ref_a).max() <= ATTN_ATOL
        assert np.abs(bf16_out_to_f32(out_b) - ref_b).max() <= ATTN_ATOL
        b.finish(stream=side)
        torch.cuda.synchronize()
        check_state(a, oa, f"cache on the main stream, token {t}")
        check_state(b, ob, f"cache on the side stream, token {t}")
    assert a.status() == 0 and b.status() == 0


def test_deferred_eviction_single_cache_and_other_entry_points():
    # no carrier: finish(), scores(), a plain block step and destroy each complete a pending eviction
    w = get_config("toy")
    N, B = w.budget_N, w.block_B
    data = make_layer(w, seed=48)
    cache, oc = make_pair(w, N, B, layout=kd.LAYOUT_FILL)
    for i, (t, Bt, q, k, v) in enumerate(blocks(data, B)):
        if i % 2 == 0:
            out = cache.prefill_block_deferred(to_dev(q), to_dev(k), to_dev(v), t)
        else:
            out = cache.prefill_block(to_dev(q), to_dev(k), to_dev(v), t)   # finishes the pending one first
        ref, _, ev = oc.prefill_block(q, k, v, t)
        assert np.abs(bf16_out_to_f32(out) - ref).max() <= ATTN_ATOL
        if i % 4 == 0:
            cache.finish()
            cache.finish()   # nothing pending: a no-op
        if i % 4 == 2 and ev > 0:
            sc = cache.scores().cpu().numpy()
            osc = oc.scores()
            order = np.argsort(cache.positions().cpu().numpy(), axis=-1, kind="stable")
            assert np.allclose(np.take_along_axis(sc, order, axis=-1), osc, rtol=SCORE_RTOL, atol=SCORE_ATOL)
        check_state(cache, oc, f"block {i}")
    with pytest.raises(kd.KeyDiffError):
        cache.prefill_block_deferred(to_dev(q), to_dev(k), to_dev(v), t + Bt, carry=cache)
    assert cache.status() == 0
    cache.close()


# ---- rotary embedding inside the call (Fig. 1 step 1, the part of it behind this boundary) ----
def rotated_reference(w, data_u, T):
    """What the rope entry points must produce from unrotated bf16 q / k: the input recipe's rotation
    (float32, every product and sum rounded on its own) of those very values, rounded once to bf16."""
    cos, sin = rope_tables(0, T, w.head_dim, w.rope_theta)
    ref = dict(data_u)
    for x in ("q", "k"):
        ref[x] = f32_to_bf16_bits(apply_rope(bf16_bits_to_f32(data_u[x]), cos, sin))
    return ref, torch.from_numpy(cos).cuda(), torch.from_numpy(sin).cuda()


@pytest.mark.parametrize("layout", [kd.LAYOUT_ORDERED, kd.LAYOUT_FILL])
@pytest.mark.parametrize("hq,hkv,d,N,B,T", [(6, 2, 128, 200, 48, 500), (8, 2, 64, 130, 100, 650)])
def test_rope_entry_point_rotates_like_the_input_recipe(layout, hq, hkv, d, N, B, T):
    # the oracle gets the block rotated by the recipe's own routine; the library gets it unrotated plus the
    # tables.  The rotated keys are compared bit for bit through the cache rows they become (check_state),
    # the rotated queries through the attention output.
    w = get_config("llama32_3b").small(n_q_heads=hq, n_kv_heads=hkv, head_dim=d, prompt_T=T)
    data_u = make_layer(w, seed=77, rotate=False)
    ref, cos, sin = rotated_reference(w, data_u, T)
    assert not np.array_equal(ref["k"], data_u["k"])
    cache, oc = make_pair(w, N, B, layout=layout)
    for (t, Bt, q, k, v), (_, _, qr, kr, _) in zip(blocks(data_u, B), blocks(ref, B)):
        out = cache.prefill_block_rope(to_dev(q), to_dev(k), to_dev(v), t, cos, sin)
        want, _, _ = oc.prefill_block(qr, kr, v, t)
        err = float(np.abs(bf16_out_to_f32(out) - want).max())
        assert err <= ATTN_ATOL, f"attention error {err} in block at token {t}"
        check_state(cache, oc, f"rope, block at token {t}")
    assert cache.status() == 0
    # a block that runs past the tables is refused before anything is enqueued
    with pytest.raises(kd.KeyDiffError) as e:
        cache.prefill_block_rope(to_dev(q), to_dev(k), to_dev(v), T, cos, sin)
    assert e.value.code == -2
    check_state(cache, oc, "after the refused call")
    cache.close()


def test_rope_through_the_layers_call():
    w = get_config("llama31_8b").small(n_q_heads=8, n_kv_heads=2, prompt_T=1280)
    N, B, L = 512, 128, 3
    raws = [make_layer(w, seed=81 + l, layer=l, rotate=False) for l in range(L)]
    refs = []
    for r in raws:
        ref, cos, sin = rotated_reference(w, r, w.prompt_T)
        refs.append(ref)
    pairs = [make_pair(w, N, B, layout=kd.LAYOUT_FILL) for _ in range(L)]
    for steps_u, steps_r in zip(zip(*(blocks(r, B) for r in raws)), zip(*(blocks(r, B) for r in refs))):
        t = steps_u[0][0]
        outs = kd.prefill_block_layers([c for c, _ in pairs], [to_dev(s_[2]) for s_ in steps_u], [to_dev(s_[3]) for s_ in steps_u],
                                       [to_dev(s_[4]) for s_ in steps_u], t, rope=(cos, sin))
        for l, (c, oc) in enumerate(pairs):
            want, _, _ = oc.prefill_block(steps_r[l][2], steps_r[l][3], steps_r[l][4], t)
            err = float(np.abs(bf16_out_to_f32(outs[l]) - want).max())
            assert err <= ATTN_ATOL, f"attention error {err}, layer {l}, block at token {t}"
    for l, (c, oc) in enumerate(pairs):
        check_state(c, oc, f"layer {l} at the end")
        assert c.status() == 0
        c.close()


def test_very_large_logits_stay_finite():
    # queries x 16 and keys x 8 (exact in bf16): logits 128 times larger, softmax close to an arg-max and
    # reference maxima that jump by hundreds between tiles -- the lazy rescale must keep everything finite
    w = get_config("llama31_8b").small(n_q_heads=8, n_kv_heads=2, prompt_T=1024)
    data = make_layer(w, seed=63)
    def scaled(bits, by):   # multiply bf16 bit patterns by a power of two: add to the exponent field
        e = (bits >> 7) & 0xFF
        out = bits.copy()
        nz = e != 0
        out[nz] = (bits[nz] & 0x807F) | (((e[nz].astype(np.int32) + by).clip(1, 254).astype(np.uint16)) << 7)
        return out
    data = dict(data, q=scaled(data["q"], 4), k=scaled(data["k"], 3))
    cache, oc = make_pair(w, 512, 128, layout=kd.LAYOUT_FILL)
    for t, Bt, q, k, v in blocks(data, 128):
        out = cache.prefill_block(to_dev(q), to_dev(k), to_dev(v), t)
        ref, _, _ = oc.prefill_block(q, k, v, t)
        got = bf16_out_to_f32(out)
        assert np.isfinite(got).all(), t
        assert np.abs(got - ref).max() <= ATTN_ATOL, t
        check_state(cache, oc, f"token {t}")
    assert cache.status() == 0


def test_values_up_to_the_documented_magnitude_limit():
    # Split-KV partial outputs are stored as fp16 (normalised by their own row sum, so bounded by the
    # largest |v| of the rows they cover): keydiff.h limits |v| to 65504.  Values scaled by 2^13 (exact in
    # bf16; the largest is then about 3.7e4, just inside the limit) must give 2^13 times the outputs of
    # the unscaled run: every rounding on the way (bf16 weights, fp16 partials, bf16 output) is scale
    # free as long as nothing overflows -- up to one bf16 step where a partial of the unscaled run was
    # an fp16 subnormal.  Through the split path, several key splits.
    w = get_config("llama31_8b").small(n_q_heads=8, n_kv_heads=2, prompt_T=1024)
    data = make_layer(w, seed=64)
    e = (data["v"] >> 7) & 0xFF
    big = data["v"].copy()
    nz = e != 0
    big[nz] = (data["v"][nz] & 0x807F) | ((e[nz].astype(np.int32) + 13).astype(np.uint16) << 7)
    vmax = float(np.abs(bf16_out_to_f32(to_dev(big))).max())
    assert 3.0e4 < vmax < 65504.0
    a, _ = make_pair(w, 512, 128, layout=kd.LAYOUT_FILL)
    b, _ = make_pair(w, 512, 128, layout=kd.LAYOUT_FILL)
    for (t, Bt, q, k, v), (_, _, _, _, vb) in zip(blocks(data, 128), blocks(dict(data, v=big), 128)):
        out_a = bf16_out_to_f32(a.prefill_block(to_dev(q), to_dev(k), to_dev(v), t))
        out_b = bf16_out_to_f32(b.prefill_block(to_dev(q), to_dev(k), to_dev(vb), t))
        assert np.isfinite(out_b).all(), t
        assert np.allclose(out_b / 8192.0, out_a, rtol=2.0 ** -7, atol=1e-4), f"outputs do not scale at token {t}"
    assert a.status() == 0 and b.status() == 0


def test_zero_key_and_tiny_keys_hit_the_eps_clamp():
    hq, hkv, d, N, B = 2, 1, 64, 40, 16
    w = get_config("toy").small(n_q_heads=hq, n_kv_heads=hkv, head_dim=d, prompt_T=64)
    data = make_layer(w, seed=4)
    k = data["k"].copy()
    k[5] = 0                                    # a zero key: score 0 by the clamp
    k[9] = f32_to_bf16_bits(np.full((hkv, d), 2.0 ** -40, dtype=np.float32))
    data = dict(data, k=k)
    run_prompt(w, data, N, B, layout=kd.LAYOUT_FILL)


def test_scores_entry_point_matches_oracle_and_leaves_the_cache_alone():
    w = get_config("llama32_3b").small(n_q_heads=6, n_kv_heads=2, prompt_T=300)
    data = make_layer(w, seed=6)
    cache, oc = make_pair(w, 256, 50, layout=kd.LAYOUT_FILL)
    for t, Bt, q, k, v in blocks(data, 50):
        cache.prefill_block(to_dev(q), to_dev(k), to_dev(v), t)
        oc.prefill_block(q, k, v, t)
    before = rows_by_position(cache)
    got = cache.scores().cpu().numpy()
    order = np.argsort(cache.positions().cpu().numpy(), axis=-1, kind="stable")
    assert np.allclose(np.take_along_axis(got, order, -1), oc.scores(), rtol=SCORE_RTOL, atol=SCORE_ATOL)
    after = rows_by_position(cache)
    assert all(np.array_equal(a, b) for a, b in zip(before, after))


def test_cache_load_resumes_from_an_oracle_state():
    w = get_config("llama32_3b").small(n_q_heads=6, n_kv_heads=2, prompt_T=400)
    data = make_layer(w, seed=8)
    N, B = 192, 64
    oc = oracle.OracleCache(1, 6, 2, 128, N, B)
    it = list(blocks(data, B))
    for t, Bt, q, k, v in it[:4]:
        oc.prefill_block(q, k, v, t)
    cache = kd.KeyDiffCache(kd.KeyDiffConfig(1, 6, 2, 128, N, B, layout=kd.LAYOUT_ORDERED))
    cache.load(to_dev(oc.keys()), to_dev(oc.values()), torch.from_numpy(oc.positions()).cuda())
    check_state(cache, oc, "after load")
    for t, Bt, q, k, v in it[4:]:
        out = cache.prefill_block(to_dev(q), to_dev(k), to_dev(v), t)
        ref, _, _ = oc.prefill_block(q, k, v, t)
        assert np.abs(bf16_out_to_f32(out) - ref).max() <= ATTN_ATOL
        check_state(cache, oc, f"resumed, token {t}")


def test_argument_errors_enqueue_nothing():
    w = get_config("toy")
    cache = kd.KeyDiffCache(kd.KeyDiffConfig(1, 4, 1, 64, 64, 16))
    q = torch.zeros((1, 4, 32, 64), dtype=torch.bfloat16, device="cuda")
    kv = torch.zeros((1, 1, 32, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(kd.KeyDiffError) as e:
        cache.prefill_block(q, kv, kv, 0)          # Bt = 32 > block_B = 16
    assert e.value.code == kd.binding.ESHAPE and cache.len == 0
    with pytest.raises(kd.KeyDiffError) as e:
        cache.scores()                              # empty cache
    assert e.value.code == kd.binding.ESTATE
    lib = kd.load_library()
    assert lib.keydiff_prefill_block(cache._h, None, None, None, 1, 0, None, None, None) == kd.binding.EINVAL
    assert cache.len == 0 and cache.status() == 0
