"""Pins for the oracle's digest and block-importance score (CPU only).

Digest: Sec. 2.2 (channel-wise min/max pooling).  Score: Sec. 2.2 / 3.2 (query
against the digest; upper bound of q.k over the block).
"""
import numpy as np
import pytest

import oracle
from paper_2603_27138_amd import workload as W


def _rand(shape, seed, dtype):
    x = np.random.default_rng(seed).standard_normal(shape).astype(np.float32)
    return W.to_storage(x, dtype)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("ctx,S,d", [(2048, 16, 64), (1000, 32, 128), (33, 32, 8), (5, 16, 4)])
def test_digest_is_array_minmax(dtype, ctx, S, d):
    K = _rand((ctx, d), 1, dtype)
    dig = oracle.digest(K, ctx, S)
    nb = (ctx + S - 1) // S
    Kf = W.storage_to_f32(K).astype(np.float64)
    pad = np.full((nb * S, d), np.nan)
    pad[:ctx] = Kf
    pad = pad.reshape(nb, S, d)
    df = W.storage_to_f32(dig).astype(np.float64)
    assert np.array_equal(df[:, 0], np.nanmin(pad, axis=1))
    assert np.array_equal(df[:, 1], np.nanmax(pad, axis=1))


def test_digest_min_le_max_and_order_matters():
    K = _rand((64, 8), 2, "f32")
    dig = oracle.digest(K, 64, 16)
    assert (dig[:, 0] <= dig[:, 1]).all()
    assert (dig[:, 0] < dig[:, 1]).any()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_score_upper_bounds_every_token(dtype):
    G, d, S, nb = 4, 64, 16, 24
    q = _rand((G, d), 3, dtype)
    K = _rand((nb * S, d), 4, dtype)
    s_heads = np.stack([oracle.score(q[h:h + 1], oracle.digest(K, nb * S, S)) for h in range(G)])
    logits = W.storage_to_f32(q).astype(np.float64) @ W.storage_to_f32(K).astype(np.float64).T   # [G][tokens]
    best = logits.reshape(G, nb, S).max(axis=2)
    assert (s_heads >= best - 1e-12).all()
    # not vacuous: the bound is within the range a min/max box allows, and strict somewhere
    assert (s_heads > best).any()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_score_single_token_block_is_plain_dot(dtype):
    G, d, nb = 3, 32, 17
    q = _rand((G, d), 5, dtype)
    K = _rand((nb, d), 6, dtype)
    s = oracle.score(q, oracle.digest(K, nb, 1))
    want = (W.storage_to_f32(q).astype(np.float64) @ W.storage_to_f32(K).astype(np.float64).T).sum(axis=0)
    np.testing.assert_allclose(s, want, rtol=1e-13, atol=1e-12)


def test_score_constant_block_is_plain_dot():
    G, d, S = 2, 16, 8
    q = _rand((G, d), 7, "f32")
    row = _rand((1, d), 8, "f32")
    K = np.repeat(row, S, axis=0)
    s = oracle.score(q, oracle.digest(K, S, S))
    want = (q.astype(np.float64) @ row.astype(np.float64).T).sum()
    np.testing.assert_allclose(s[0], want, rtol=1e-13)


def test_score_translation_equivariance():
    """Shifting every key of a block by u adds sum_h q_h.u to its score, exactly in real arithmetic."""
    G, d, S, nb = 4, 32, 16, 6
    rng = np.random.default_rng(9)
    # small dyadic values so that the shifted keys are exact in float32
    q = (rng.integers(-8, 9, (G, d)) / 8.0).astype(np.float32)
    K = (rng.integers(-64, 65, (nb * S, d)) / 16.0).astype(np.float32)
    u = (rng.integers(-16, 17, d) / 4.0).astype(np.float32)
    s0 = oracle.score(q, oracle.digest(K, nb * S, S))
    K2 = K.copy()
    K2[2 * S:3 * S] += u
    s1 = oracle.score(q, oracle.digest(K2, nb * S, S))
    shift = (q.astype(np.float64) @ u.astype(np.float64)).sum()
    want = s0.copy()
    want[2] += shift
    np.testing.assert_allclose(s1, want, rtol=0, atol=1e-10)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_score_group_is_sum_of_heads_and_folded_form(dtype):
    G, d, S, nb = 8, 128, 32, 40
    q = _rand((G, d), 10, dtype)
    K = _rand((nb * S, d), 11, dtype)
    dig = oracle.digest(K, nb * S, S)
    s = oracle.score(q, dig)
    per_head = sum(oracle.score(q[h:h + 1], dig) for h in range(G))
    np.testing.assert_allclose(s, per_head, rtol=1e-13)
    # folded form: P = sum of positive parts, N = sum of negative parts of the group's queries
    qf = W.storage_to_f32(q).astype(np.float64)
    df = W.storage_to_f32(dig).astype(np.float64)
    P, N = np.clip(qf, 0, None).sum(0), np.clip(qf, None, 0).sum(0)
    folded = df[:, 1] @ P + df[:, 0] @ N
    np.testing.assert_allclose(s, folded, rtol=1e-12)


def test_score_sign_handling_tiny_by_hand():
    # one block, two tokens, d = 2: k0 = (1, -2), k1 = (3, 4); min = (1,-2), max = (3,4)
    K = np.array([[1, -2], [3, 4]], dtype=np.float32)
    q = np.array([[2, -1]], dtype=np.float32)
    # channel 0: max(2*1, 2*3) = 6; channel 1: max(-1*-2, -1*4) = 2  -> 8
    assert oracle.score(q, oracle.digest(K, 2, 2))[0] == 8.0
    q2 = np.array([[2, -1], [-1, 1]], dtype=np.float32)
    # second head: channel 0: max(-1, -3) = -1; channel 1: max(-2, 4) = 4 -> 3 ; group 11
    assert oracle.score(q2, oracle.digest(K, 2, 2))[0] == 11.0


def test_planted_blocks_rank_high_on_tiny():
    wl = W.generate(W.tiny())
    dig = oracle.digest(wl.K[(0, 0)], 2048, 16)
    s = oracle.score(wl.q[0], dig)
    top = set(oracle.select(s, 16).tolist())
    assert len(top & set(wl.planted[(0, 0)].tolist())) >= 7


# ---------------------------------------------------------------- max over the group's heads

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("G,d,nb,S", [(8, 128, 9, 32), (4, 64, 5, 16), (16, 8, 3, 4)])
def test_score_max_is_the_maximum_of_the_per_head_estimates(dtype, G, d, nb, S):
    K = _rand((nb * S, d), 21, dtype)
    q = _rand((G, d), 22, dtype)
    dig = oracle.digest(K, nb * S, S)
    qf = W.storage_to_f32(q).astype(np.float64)
    df = W.storage_to_f32(dig).astype(np.float64)
    per_head = np.maximum(qf[None, :, :] * df[:, None, 0, :], qf[None, :, :] * df[:, None, 1, :]).sum(-1)   # [nb][G]
    got = oracle.score_max(q, dig)
    assert np.allclose(got, per_head.max(axis=1), rtol=1e-13, atol=0)
    # the sum over heads is the other aggregation: never below the maximum when every estimate is positive,
    # and equal to it for a group of one head
    assert np.allclose(oracle.score(q, dig), per_head.sum(axis=1), rtol=1e-13, atol=0)
    assert np.array_equal(oracle.score_max(q[:1], dig), oracle.score(q[:1], dig))
    # each head's estimate bounds its dot products over the block from above, so does the maximum for its own head
    Kf = W.storage_to_f32(K).astype(np.float64).reshape(nb, S, d)
    dots = np.einsum("hc,jtc->jht", qf, Kf).max(axis=2)     # [nb][G] largest true logit per head
    assert (per_head >= dots - 1e-9).all() and (got >= dots.max(axis=1) - 1e-9).all()


# ---------------------------------------------------------------- mean-pooled digest (stored as sums)

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("ctx,S", [(96, 32), (70, 16), (5, 64), (64, 64)])
def test_digest_sum_is_the_sequential_binary32_sum(dtype, ctx, S):
    rng = np.random.default_rng(ctx * 7 + S)
    K = W.to_storage(rng.standard_normal((ctx, 24)).astype(np.float32) * 3, dtype)
    got = oracle.digest_sum(K, ctx, S)
    Kf = W.storage_to_f32(K)
    nb = (ctx + S - 1) // S
    assert got.shape == (nb, 24) and got.dtype == np.float32
    for j in range(nb):
        blk = Kf[j * S:min(ctx, (j + 1) * S)]
        assert np.array_equal(got[j], np.cumsum(blk, axis=0, dtype=np.float32)[-1])      # sequential, one rounding per token
        exact = blk.astype(np.float64).sum(axis=0)
        assert np.abs(got[j] - exact).max() <= 1e-6 * np.abs(blk).astype(np.float64).sum(axis=0).max()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_append_sum_grows_the_digest_built_at_once(dtype):
    rng = np.random.default_rng(77)
    S, d, mb = 8, 16, 5
    K = W.to_storage(rng.standard_normal((mb * S, d)).astype(np.float32), dtype)
    sums = np.full((mb, d), 123.0, dtype=np.float32)       # stale contents must not leak into a new block
    for t in range(mb * S - 3):
        oracle.append_sum(S, t, K[t], sums)
        nb = t // S + 1
        assert np.array_equal(sums[:nb], oracle.digest_sum(K[:t + 1], t + 1, S)), t
    before = sums.copy()
    oracle.append_sum(S, mb * S, K[0], sums)                # a full sequence is left as it is
    assert np.array_equal(sums, before)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_score_mean_is_the_query_group_against_the_block_means(dtype):
    rng = np.random.default_rng(91)
    ctx, S, d, G = 150, 32, 64, 4
    K = W.to_storage(rng.standard_normal((ctx, d)).astype(np.float32), dtype)
    q = W.to_storage(rng.standard_normal((G, d)).astype(np.float32), dtype)
    sums = oracle.digest_sum(K, ctx, S)
    got = oracle.score_mean(q, sums, ctx, S)
    Kf, qf = W.storage_to_f32(K).astype(np.float64), W.storage_to_f32(q).astype(np.float64)
    for j in range(len(sums)):
        blk = Kf[j * S:min(ctx, (j + 1) * S)]
        want = float((qf @ blk.mean(axis=0)).sum())         # sum over heads of q_h . mean_j, exact means
        assert abs(got[j] - want) <= 1e-5 * max(1.0, abs(want)), j
        # and exactly the definition on the stored sums
        want2 = float((qf @ sums[j].astype(np.float64)).sum()) / len(blk)
        assert abs(got[j] - want2) <= 1e-12 * max(1.0, abs(want2))
    # a transposed operand or a forgotten division by the count of the partly filled last block would show
    assert ctx % S != 0
