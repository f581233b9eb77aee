"""Pins for the oracle's partial attention and merge (CPU only).

Partial attention: Sec. 3.2 (each side attends to its share of the selected
blocks).  Merge: Algorithm 1, Merge step (FlashAttention rescaling).
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_27138_amd import workload as W
from tests import harness


def _rand(shape, seed, dtype="f32", scale=1.0):
    x = (np.random.default_rng(seed).standard_normal(shape) * scale).astype(np.float32)
    return W.to_storage(x, dtype)


def _f64(a):
    return W.storage_to_f32(a).astype(np.float64)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("ctx,S", [(256, 16), (250, 32), (31, 32)])
def test_all_blocks_equals_library_dense_attention(dtype, ctx, S):
    """k covering every block, everything resident: the partial IS dense attention (torch SDPA, fp64)."""
    G, d = 4, 64
    q, K, V = _rand((G, d), 1, dtype), _rand((ctx, d), 2, dtype), _rand((ctx, d), 3, dtype)
    nb = (ctx + S - 1) // S
    scale = 1.0 / np.sqrt(d)
    tq = torch.from_numpy(_f64(q))[None, :, None, :]                   # [1][G][1][d]
    tk = torch.from_numpy(_f64(K))[None, None].expand(1, G, ctx, d)    # KV head repeated G times
    tv = torch.from_numpy(_f64(V))[None, None].expand(1, G, ctx, d)
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, scale=scale)[0, :, 0].numpy()
    lse_want = torch.logsumexp(torch.from_numpy(_f64(q) @ _f64(K).T * scale), dim=1).numpy()
    for h in range(G):
        o, m, l = oracle.partial_attn(q[h], K, V, np.arange(nb), ctx, S, scale)
        np.testing.assert_allclose(o, want[h], rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(m + np.log(l), lse_want[h], rtol=1e-13)


def test_sparse_subset_equals_dense_over_those_tokens():
    G, d, S, nb = 2, 32, 16, 10
    q, K, V = _rand((G, d), 4), _rand((nb * S, d), 5), _rand((nb * S, d), 6)
    blocks = [7, 1, 4]
    tok = np.concatenate([np.arange(j * S, (j + 1) * S) for j in blocks])
    scale = 0.3
    p = torch.softmax(torch.from_numpy(_f64(q) @ _f64(K)[tok].T * scale), dim=1).numpy()
    want = p @ _f64(V)[tok]
    for h in range(G):
        o, _, _ = oracle.partial_attn(q[h], K, V, blocks, nb * S, S, scale)
        np.testing.assert_allclose(o, want[h], rtol=1e-12, atol=1e-13)


def test_weights_sum_to_one():
    d, S, nb = 16, 8, 6
    q, K = _rand((1, d), 7), _rand((nb * S, d), 8)
    ones = np.ones((nb * S, d), dtype=np.float32)
    o, _, _ = oracle.partial_attn(q[0], K, ones, [0, 3, 5], nb * S, S, 0.25)
    np.testing.assert_allclose(o, 1.0, rtol=1e-14)
    c = _rand((1, d), 9)
    o, _, _ = oracle.partial_attn(q[0], K, np.repeat(c, nb * S, 0), [1, 2], nb * S, S, 0.25)
    np.testing.assert_allclose(o, c[0].astype(np.float64), rtol=1e-14)


def test_closed_forms():
    d, S = 8, 4
    q = _rand((1, d), 10)
    # all keys equal: uniform weights, l = token count, m = scale * q.k
    k = _rand((1, d), 11)
    K = np.repeat(k, 3 * S, 0)
    V = _rand((3 * S, d), 12)
    o, m, l = oracle.partial_attn(q[0], K, V, [0, 2], 3 * S, S, 0.5)
    np.testing.assert_allclose(o, np.concatenate([V[:S], V[2 * S:]]).astype(np.float64).mean(0), rtol=1e-13)
    assert l == pytest.approx(2 * S, rel=1e-14)
    assert m == pytest.approx(0.5 * float(q[0].astype(np.float64) @ k[0].astype(np.float64)), rel=1e-14)
    # two tokens whose logits differ by ln 3: weights 3/4 and 1/4
    q2 = np.array([1.0, 0.0], dtype=np.float32)
    K2 = np.array([[np.log(3.0), 5.0], [0.0, -7.0]], dtype=np.float32)
    V2 = np.array([[4.0, 0.0], [0.0, 8.0]], dtype=np.float32)
    o, m, l = oracle.partial_attn(q2, K2, V2, [0], 2, 2, 1.0)
    np.testing.assert_allclose(o, [3.0, 2.0], rtol=1e-7)
    assert m == pytest.approx(float(np.float32(np.log(3.0))))
    assert l == pytest.approx(1.0 + 1.0 / 3.0, rel=1e-7)
    # one dominant key: output tends to its value
    K3 = np.zeros((4, 2), dtype=np.float32)
    K3[2, 0] = 100.0
    V3 = _rand((4, 2), 13)
    o, _, _ = oracle.partial_attn(q2, K3, V3, [0], 4, 4, 1.0)
    np.testing.assert_allclose(o, V3[2].astype(np.float64), atol=1e-40)


def test_empty_set_and_masked_tail():
    d, S = 8, 4
    q, K, V = _rand((1, d), 14), _rand((10, d), 15), _rand((10, d), 16)
    o, m, l = oracle.partial_attn(q[0], K, V, [], 10, S, 1.0)
    assert (o == 0).all() and m == -np.inf and l == 0
    # last block has 2 valid tokens of 4: equals attention over tokens 8, 9 only
    o, m, l = oracle.partial_attn(q[0], K, V, [2], 10, S, 1.0)
    x = K[8:10].astype(np.float64) @ q[0].astype(np.float64)
    p = np.exp(x - x.max())
    np.testing.assert_allclose(o, p @ V[8:10].astype(np.float64) / p.sum(), rtol=1e-13)


def test_block_order_invariance_and_gqa_equals_mha():
    G, d, S, nb = 4, 32, 16, 8
    q, K, V = _rand((G, d), 17), _rand((nb * S, d), 18), _rand((nb * S, d), 19)
    a = oracle.partial_attn(q[1], K, V, [1, 4, 6], nb * S, S, 0.2)
    b = oracle.partial_attn(q[1], K, V, [6, 1, 4], nb * S, S, 0.2)
    np.testing.assert_allclose(a[0], b[0], rtol=1e-13)
    assert a[1] == b[1] and a[2] == pytest.approx(b[2], rel=1e-14)
    # MHA with the KV head copied per query head is the same computation per head
    for h in range(G):
        c = oracle.partial_attn(q[h], K.copy(), V.copy(), [1, 4, 6], nb * S, S, 0.2)
        e = oracle.partial_attn(q[h], K, V, [1, 4, 6], nb * S, S, 0.2)
        assert np.array_equal(c[0], e[0])


# ------------------------------------------------------------------------ merge


@pytest.mark.parametrize("seed", range(10))
def test_merge_of_any_split_is_attention_over_union(seed):
    rng = np.random.default_rng(seed)
    d, S, nb = 16, 8, 12
    q, K, V = _rand((1, d), 100 + seed, scale=2.0), _rand((nb * S, d), 200 + seed), _rand((nb * S, d), 300 + seed)
    T = rng.permutation(nb)[:7]
    cut = rng.integers(0, 8)
    A, Bs = T[:cut], T[cut:]
    pa = oracle.partial_attn(q[0], K, V, A, nb * S, S, 0.7)
    pb = oracle.partial_attn(q[0], K, V, Bs, nb * S, S, 0.7)
    pu = oracle.partial_attn(q[0], K, V, T, nb * S, S, 0.7)
    out, lse = oracle.merge(*pa, *pb)
    np.testing.assert_allclose(out, pu[0], rtol=1e-12, atol=1e-14)
    assert lse == pytest.approx(pu[1] + np.log(pu[2]), rel=1e-13)


def test_merge_identity_commutative_associative_shift():
    d = 8
    rng = np.random.default_rng(5)
    a = (rng.standard_normal(d), 1.3, 4.0)
    b = (rng.standard_normal(d), -0.4, 2.5)
    c = (rng.standard_normal(d), 7.0, 0.1)
    e = (np.zeros(d), -np.inf, 0.0)
    out, lse = oracle.merge(*a, *e)
    np.testing.assert_allclose(out, a[0], rtol=1e-15)
    assert lse == pytest.approx(a[1] + np.log(a[2]))
    out2, lse2 = oracle.merge(*e, *a)
    np.testing.assert_allclose(out2, a[0], rtol=1e-15)
    o0, l0 = oracle.merge(*e, *e)
    assert (o0 == 0).all() and l0 == -np.inf
    ab, ba = oracle.merge(*a, *b), oracle.merge(*b, *a)
    np.testing.assert_allclose(ab[0], ba[0], rtol=1e-15)
    assert ab[1] == pytest.approx(ba[1], rel=1e-15)
    # associativity: ((a,b),c) == (a,(b,c)), carrying the merged pair as (o, lse, 1)
    left = oracle.merge(ab[0], ab[1], 1.0, *c)
    bc = oracle.merge(*b, *c)
    right = oracle.merge(*a, bc[0], bc[1], 1.0)
    np.testing.assert_allclose(left[0], right[0], rtol=1e-13)
    assert left[1] == pytest.approx(right[1], rel=1e-14)
    # (o, m + delta, l * exp(-delta)) is the same partial
    delta = 2.25
    sh = oracle.merge(a[0], a[1] + delta, a[2] * np.exp(-delta), *b)
    np.testing.assert_allclose(sh[0], ab[0], rtol=1e-13)
    assert sh[1] == pytest.approx(ab[1], rel=1e-14)
    # weights by hand: m equal, l 1 and 3 -> 1/4, 3/4
    o, lse = oracle.merge(np.full(d, 4.0), 0.0, 1.0, np.full(d, 8.0), 0.0, 3.0)
    np.testing.assert_allclose(o, 7.0)
    assert lse == pytest.approx(np.log(4.0))


def test_pipeline_on_tiny_dense_equals_sparse_when_k_covers_all():
    """Whole chain on config 1 with k = all blocks and nothing offloaded equals dense attention."""
    cfg = W.shrink(W.tiny(), k=128)
    wl = W.generate(cfg)
    op = harness.run_pair(wl, 0, 0)
    assert op.n_gpu == 128 and op.n_host == 0
    K, V = wl.K[(0, 0)].astype(np.float64), wl.V[(0, 0)].astype(np.float64)
    q = wl.q[0].astype(np.float64)
    p = torch.softmax(torch.from_numpy(q @ K.T * cfg.sm_scale), dim=1).numpy()
    want = p @ V
    for h in range(cfg.G):
        np.testing.assert_allclose(op.out[h][0], want[h], rtol=1e-12, atol=1e-14)


def test_pipeline_merge_equals_union_on_split_residency():
    cfg = W.shrink(W.tiny(), p_host=0.5)
    wl = W.generate(cfg)
    op = harness.run_pair(wl, 0, 0)
    assert op.n_gpu + op.n_host == cfg.k and op.n_host > 0 and op.n_gpu > 0
    qg = wl.q[0]
    for h in range(cfg.G):
        pu = oracle.partial_attn(qg[h], wl.K[(0, 0)], wl.V[(0, 0)], op.sel, 2048, cfg.S, cfg.sm_scale)
        np.testing.assert_allclose(op.out[h][0], pu[0], rtol=0, atol=1e-6)   # host partial went through binary32


def test_per_head_selection_is_the_brute_force_rule_per_head():
    """Selection per query head: every head keeps the k blocks with the largest value of ITS OWN
    estimate sum_c max(q_c*min_c, q_c*max_c) (ties to the lower index), attends to exactly those, and
    heads of one KV head may differ in what they keep."""
    cfg = W.shrink(W.qwen3_8b(B=1, ctx=2048), p_host=0.5, k=8)
    wl = W.generate(cfg)
    differ = False
    for hq in range(cfg.Hq):
        op = harness.run_head(wl, 0, hq)
        g = hq // cfg.G
        q = _f64(wl.q[0, hq])
        dig = _f64(op.dig)
        est = np.maximum(q * dig[:, 0], q * dig[:, 1]).sum(axis=1)
        est32 = est.astype(np.float32).astype(np.float64)
        want = sorted(sorted(range(len(est)), key=lambda j: (-est32[j], j))[:cfg.k])
        assert [int(j) for j in op.sel if j >= 0] == want, hq
        # the two sides split that list by the KV head's residency and their merge is the attention over it
        assert sorted(op.sel_gpu[:op.n_gpu].tolist() + op.sel_host[:op.n_host].tolist()) == want
        assert all(wl.block_table[0, g, j] >= 0 for j in op.sel_gpu[:op.n_gpu])
        pu = oracle.partial_attn(wl.q[0, hq], wl.K[(0, g)], wl.V[(0, g)], op.sel, int(cfg.ctx[0]), cfg.S, cfg.sm_scale)
        np.testing.assert_allclose(op.out[0][0], pu[0], rtol=0, atol=1e-6)
        shared = harness.run_pair(wl, 0, g, attention=False)
        differ |= not np.array_equal(shared.sel, op.sel)
    assert differ   # otherwise this workload could not tell the variant from the shared selection
