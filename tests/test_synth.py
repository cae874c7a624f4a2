"""The seeded generator: determinism, random access by token range, shapes."""
import numpy as np

from synth import bf16_bits_to_f32, block_of, f32_to_bf16_bits, get_config, make_layer


def test_bf16_rounding_is_nearest_even_and_round_trips():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 0.0, 3.140625], dtype=np.float32)
    b = f32_to_bf16_bits(x)
    back = bf16_bits_to_f32(b)
    # 1 + 2^-8 is a tie between 1 and 1 + 2^-7: goes to the even mantissa (1.0);
    # 1 + 3*2^-8 ties between 1+2^-7 (odd) and 1+2^-6 (even): goes up
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == 1.015625
    assert np.array_equal(f32_to_bf16_bits(back), b)


def test_same_seed_same_bits_and_token_ranges_are_random_access():
    w = get_config("llama32_3b").small(prompt_T=700)
    a = make_layer(w, seed=5, layer=2)
    b = make_layer(w, seed=5, layer=2)
    part = make_layer(w, seed=5, layer=2, t0=300, t1=650)
    for key in ("q", "k", "v"):
        assert np.array_equal(a[key], b[key])
        assert np.array_equal(a[key][300:650], part[key])
    c = make_layer(w, seed=5, layer=3)
    assert not np.array_equal(a["k"], c["k"])


def test_shapes_layout_and_outlier_rate():
    w = get_config("qwen25_7b").small(prompt_T=512)
    data = make_layer(w, seed=9)
    assert data["q"].shape == (512, 28, 128) and data["k"].shape == (512, 4, 128)
    blk = block_of(data["k"], 256, 256)
    assert blk.shape == (4, 256, 128) and blk.flags["C_CONTIGUOUS"]
    assert np.array_equal(blk[2, 7], data["k"][263, 2])
    toy = get_config("toy")
    k = bf16_bits_to_f32(make_layer(toy, seed=1)["k"])[:, 0]
    norms = np.linalg.norm(k, axis=1)
    frac = np.mean(norms > 2.5 * np.median(norms))
    assert 0.005 < frac < 0.05          # about 2 % of keys are scaled x4
