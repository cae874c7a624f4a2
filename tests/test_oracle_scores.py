"""Pins for the oracle's anchor, score and selection (CPU only).

Each test fixes the oracle to something other than itself: a closed form worked
by hand, a library routine, an identity the paper derives, an invariance of the
cosine, or brute force on a tiny input.
"""
import math

import numpy as np
import pytest

import oracle
from oracle import opcount
from synth import bf16_bits_to_f64, f32_to_bf16_bits


def bits(x):
    return f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def rand_keys(rng, n, d, offset=1.0):
    return bits(rng.standard_normal((n, d)) + offset * rng.standard_normal(d))


# ----------------------------------------------------------------- hand examples
def test_two_orthogonal_keys_closed_form():
    # keys (1,0), (0,1): anchor (.5,.5), both cosines 1/sqrt 2
    s64, s32 = oracle.scores(bits([[1, 0], [0, 1]]))
    assert np.allclose(s64, 1 / math.sqrt(2), rtol=0, atol=1e-15)
    assert s32.dtype == np.float32 and np.all(s32 == np.float32(1 / math.sqrt(2)))


def test_unequal_keys_closed_form_and_kept_key():
    # keys (3,0), (0,1): anchor (1.5,.5) -> cosines 3/sqrt10 and 1/sqrt10.
    K = bits([[3, 0], [0, 1]])
    mu = oracle.anchor(K)
    assert np.array_equal(mu, [1.5, 0.5])
    s64, s32 = oracle.scores(K)
    assert np.allclose(s64, [3 / math.sqrt(10), 1 / math.sqrt(10)], rtol=0, atol=1e-15)
    # Fig. 3 (3): the LOWEST similarity is retained -> key #2 survives a budget of one
    kept = oracle.select(s32, np.array([0, 1], np.int32), keep=1)
    assert kept.tolist() == [1]


def test_unit_key_anchor_ties_and_lower_position_is_kept():
    # Eq. 7 anchor: mean of unit keys (.5,.5) -> both cosines 1/sqrt 2: a tie,
    # resolved towards the lower position.  Also tells the two anchors apart.
    K = bits([[3, 0], [0, 1]])
    assert np.allclose(oracle.anchor(K, mode=1), [0.5, 0.5])
    s64, s32 = oracle.scores(K, mode=1)
    assert s32[0] == s32[1]
    assert oracle.select(s32, np.array([0, 1], np.int32), keep=1).tolist() == [0]
    # tie-break follows position, not row order
    assert oracle.select(s32, np.array([7, 2], np.int32), keep=1).tolist() == [1]


def test_identical_keys_score_one_and_zero_key_scores_zero():
    K = bits(np.tile([[0.5, -2.0, 4.0]], (9, 1)))
    s64, _ = oracle.scores(K)
    assert np.allclose(s64, 1.0, rtol=0, atol=1e-15)
    K = bits([[1, 2, 3], [0, 0, 0], [2, 1, 0]])
    s64, s32 = oracle.scores(K)
    assert s64[1] == 0.0 and s32[1] == 0.0        # eps clamp: 0 / eps
    s64u, _ = oracle.scores(K, mode=1)            # zero key adds nothing to the unit anchor
    assert s64u[1] == 0.0 and np.all(np.isfinite(s64u))


def test_opposite_key_scores_minus_one():
    # "-1 is the extreme distinct key": a key anti-parallel to the anchor
    K = bits([[4, 0], [4, 0], [4, 0], [-2, 0]])
    s64, s32 = oracle.scores(K)
    assert np.allclose(s64, [1, 1, 1, -1], atol=1e-15)
    assert oracle.select(s32, np.arange(4, dtype=np.int32), keep=1).tolist() == [3]


def test_eps_clamps_the_product_of_norms():
    # |mu||k| = 2^-40 * ... below eps: score = dot / eps exactly
    tiny = 2.0 ** -20
    K = bits([[tiny, 0.0], [tiny, 0.0]])
    s64, _ = oracle.scores(K, eps=1e-8)
    assert np.allclose(s64, (tiny * tiny) / 1e-8, rtol=1e-15)


# ------------------------------------------------------------- library routines
def test_against_library_cosine_and_mean():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(5)
    K = rand_keys(rng, 257, 64, offset=2.0)
    Kd = torch.from_numpy(bf16_bits_to_f64(K))
    mu = Kd.mean(dim=0)
    ref = torch.nn.functional.cosine_similarity(mu[None, :], Kd, dim=1, eps=1e-12).numpy()
    s64, s32 = oracle.scores(K)
    assert np.allclose(oracle.anchor(K), mu.numpy(), rtol=1e-14, atol=0)
    assert np.allclose(s64, ref, rtol=1e-13, atol=1e-15)
    assert np.array_equal(s32, s64.astype(np.float32))
    assert np.all(np.abs(s64) <= 1 + 1e-15)


def test_non_square_shapes_catch_a_transposed_operand():
    rng = np.random.default_rng(6)
    K = rand_keys(rng, 5, 48)
    assert oracle.anchor(K).shape == (48,)
    assert oracle.scores(K)[0].shape == (5,)


# ------------------------------------------------------------------ invariances
def test_scale_rotation_and_permutation_invariance():
    rng = np.random.default_rng(7)
    n, d = 200, 32
    x = bf16_bits_to_f64(rand_keys(rng, n, d)).astype(np.float32)
    base, _ = oracle.scores(bits(x))
    # common positive scale (a power of two is exact in bf16)
    for c in (0.25, 8.0):
        s, _ = oracle.scores(bits(x * c))
        assert np.allclose(s, base, rtol=0, atol=1e-14)
    # a common orthogonal map that is exact in bf16: signed coordinate permutation
    perm = rng.permutation(d)
    sign = rng.choice([-1.0, 1.0], size=d).astype(np.float32)
    s, _ = oracle.scores(bits(x[:, perm] * sign))
    assert np.allclose(s, base, rtol=0, atol=1e-14)
    # permutation equivariance over tokens
    p = rng.permutation(n)
    s, _ = oracle.scores(bits(x[p]))
    assert np.allclose(s, base[p], rtol=0, atol=1e-14)


def test_theorem_bound_holds_for_the_cosines():
    # Theorem 3.2: cos(kbar, k*) <= 1 + a b - a^2/2 - b^2/2 with a = cos(kbar, q) < 0 < b = cos(k*, q)
    rng = np.random.default_rng(8)
    checked = 0
    for _ in range(400):
        d = int(rng.integers(2, 24))
        kbar, kstar, q = (bf16_bits_to_f64(bits(rng.standard_normal(d))) for _ in range(3))
        a = oracle.scores(bits(kbar[None]), mu=q)[0][0]
        b = oracle.scores(bits(kstar[None]), mu=q)[0][0]
        if not (a < 0 < b):
            continue
        c = oracle.scores(bits(kstar[None]), mu=kbar)[0][0]
        assert c <= 1 + a * b - 0.5 * a * a - 0.5 * b * b + 1e-12
        checked += 1
    assert checked > 40


# ------------------------------------------------- Eq. 6 (pairwise) vs Eq. 7 (anchor)
def test_unit_anchor_score_is_a_positive_multiple_of_the_pairwise_row_sum():
    # (CosSim(K) 1)_i = khat_i . sum_j khat_j = n |mu(Khat)| cos(mu(Khat), k_i)
    rng = np.random.default_rng(9)
    n, d = 300, 16
    K = rand_keys(rng, n, d, offset=0.7)
    x = bf16_bits_to_f64(K)
    xh = x / np.linalg.norm(x, axis=1, keepdims=True)
    gram_rowsum = (xh @ xh.T).sum(axis=1)                 # Eq. 6, written with a matmul
    assert np.allclose(oracle.pairwise_rowsum(K), gram_rowsum, rtol=1e-12)
    mu_hat = oracle.anchor(K, mode=1)
    s64, s32 = oracle.scores(K, mode=1)
    assert np.allclose(gram_rowsum, n * np.linalg.norm(mu_hat) * s64, rtol=1e-12)
    # hence the same retained set: topk(-CosSim(K) 1, N)
    N = 200
    want = np.sort(np.argsort(gram_rowsum, kind="stable")[:N])
    got = oracle.select(s32, np.arange(n, dtype=np.int32), keep=N)
    assert np.array_equal(got, want)


# --------------------------------------------------------------------- selection
@pytest.mark.parametrize("n,keep", [(1, 1), (2, 1), (17, 5), (64, 63), (300, 256), (40, 40), (40, 50)])
def test_select_equals_brute_force_argsort(n, keep):
    rng = np.random.default_rng(100 + n)
    # few distinct scores so that ties at the boundary are common
    s = rng.choice(np.linspace(-1, 1, 7), size=n).astype(np.float32)
    pos = rng.permutation(10 * n)[:n].astype(np.int32)
    order = np.lexsort((pos, s))                # by score, then position
    want = order[:min(keep, n)]
    want = want[np.argsort(pos[want])]
    got = oracle.select(s, pos, keep)
    assert got.shape[0] == min(keep, n)
    assert np.array_equal(got, want)
    assert np.all(np.diff(pos[got]) > 0)


def test_select_is_invariant_to_row_order():
    rng = np.random.default_rng(11)
    n, keep = 120, 77
    s = rng.choice(np.linspace(-1, 1, 9), size=n).astype(np.float32)
    pos = rng.permutation(n).astype(np.int32)
    base = set(pos[oracle.select(s, pos, keep)].tolist())
    for _ in range(5):
        p = rng.permutation(n)
        assert set(pos[p][oracle.select(s[p], pos[p], keep)].tolist()) == base


def test_sliding_window_keeps_the_most_recent_rows():
    rng = np.random.default_rng(12)
    n, keep, W = 90, 60, 12
    s = rng.standard_normal(n).astype(np.float32)
    pos = rng.permutation(n).astype(np.int32)
    kept = oracle.select(s, pos, keep, window_W=W)
    kept_pos = set(pos[kept].tolist())
    assert len(kept_pos) == keep
    assert set(range(n - W, n)) <= kept_pos                      # the W highest positions
    rest = np.nonzero(pos < n - W)[0]
    order = rest[np.lexsort((pos[rest], s[rest]))][:keep - W]    # lowest scores of the others
    assert kept_pos == set(range(n - W, n)) | set(pos[order].tolist())
    assert np.array_equal(oracle.select(s, pos, keep, window_W=0), oracle.select(s, pos, keep))


# --------------------------------------------------------------------- op counts
@pytest.mark.parametrize("n,d", [(1, 1), (7, 3), (288, 64), (8320, 128)])
def test_operation_tally_matches_the_printed_closed_form(n, d):
    ops = opcount.tally(n, d)
    assert ops == {"mul": 3 * n * d + d + n, "add": 3 * n * d - n - 1, "div": 2 * n + 2, "sqrt": n + 1}
    assert opcount.weighted(ops) == (12 * d + 97) * n + 3 * d + 94
