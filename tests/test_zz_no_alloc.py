"""keydiff_prefill_block_static (the block step with its temporaries in the library's static device
array, for callers that cannot allocate) against keydiff_prefill_block, through the C ABI.

Two handles run the same seeded prompt, one per entry point: attention outputs, scores, retained
positions and the K/V rows behind them must be identical bit for bit (same kernels, same launch
plan, only the scratch address differs).  The sequence holds full blocks followed by a smaller
one, so a call always finds the previous, larger call's contents in the array; a second
configuration then reuses the array with a different layout of its pieces.
"""
import numpy as np
import pytest

import paper_2504_15364_amd as kd
from helpers import blocks, rows_by_position, to_bits, to_dev
from synth import get_config, make_layer

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def run_pair(w, N, B, T, layout, seed):
    data = make_layer(w, seed=seed, t1=T)
    cfg = kd.KeyDiffConfig(1, w.n_q_heads, w.n_kv_heads, w.head_dim, N, B, layout=layout)
    ref, sta = kd.KeyDiffCache(cfg), kd.KeyDiffCache(cfg)
    sta._scratch.fill_(0xFF)     # the static entry point must not depend on (or touch) the handle's buffer
    torch.cuda.synchronize()
    calls = 0
    for t, Bt, q, k, v in blocks(data, B, T):
        dq, dk, dv = to_dev(q), to_dev(k), to_dev(v)
        n = ref.len + Bt
        sc_ref = torch.zeros((1, w.n_kv_heads, n), dtype=torch.float32, device="cuda")
        sc_sta = torch.zeros_like(sc_ref)
        out_ref = ref.prefill_block(dq, dk, dv, t, scores_out=sc_ref)
        out_sta = torch.empty_like(dq)
        sta.prefill_block_static(dq, dk, dv, t, out=out_sta, scores_out=sc_sta)
        assert np.array_equal(to_bits(out_ref), to_bits(out_sta)), f"attention output differs at token {t} (Bt {Bt})"
        assert torch.equal(sc_ref, sc_sta), f"scores differ at token {t}"
        pr, Kr, Vr = rows_by_position(ref)
        ps, Ks, Vs = rows_by_position(sta)
        assert np.array_equal(pr, ps) and np.array_equal(Kr, Ks) and np.array_equal(Vr, Vs), f"cache differs at token {t}"
        calls += 1
    assert ref.status() == 0 and sta.status() == 0
    assert torch.all(sta._scratch == 0xFF), "the static entry point wrote into the handle's scratch buffer"
    ref.close()
    sta.close()
    return calls


def test_static_scratch_step_matches_prefill_block_on_consecutive_calls():
    # 6 full blocks of 64 then one of 36 rows (the smaller input right after a larger one); several
    # key splits and an eviction in most steps
    w = get_config("llama32_3b").small(n_q_heads=8, n_kv_heads=2, head_dim=128, prompt_T=420)
    assert run_pair(w, 192, 64, 420, kd.LAYOUT_FILL, seed=9) == 7
    # a second, smaller configuration in the other layout reuses the same array
    w2 = get_config("toy").small(prompt_T=150)
    assert run_pair(w2, 64, 32, 150, kd.LAYOUT_ORDERED, seed=10) == 5


def test_static_scratch_rejects_a_configuration_that_does_not_fit():
    # many sequences: the score and destination-map pieces alone exceed the array
    cfg = kd.KeyDiffConfig(64, 8, 8, 64, 16384, 64)
    from paper_2504_15364_amd import binding
    assert binding.workspace_bytes(cfg)[3] > 40 << 20
    c = kd.KeyDiffCache(cfg)
    x = torch.zeros((64, 8, 64, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(kd.KeyDiffError) as e:
        c.prefill_block_static(x, x, x, 0, out=torch.empty_like(x))
    assert e.value.code == -2 and "static" in str(e.value)
    assert c.len == 0
    c.close()
