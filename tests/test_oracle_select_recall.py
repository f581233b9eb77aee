"""Pins for the oracle's top-k selection, residency split and recall plan (CPU only).

Selection: Algorithm 1 (TopK of the digest scores), ties toward the lower
block index.  Recall plan: Sec. 3.4, minimal-movement reading.
"""
import itertools

import numpy as np
import pytest

import oracle
from paper_2603_27138_amd import workload as W


def brute_topk(s, k):
    order = sorted(range(len(s)), key=lambda j: (-s[j], j))
    return sorted(order[: min(k, len(s))])


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("nb,k", [(1, 1), (7, 3), (16, 16), (16, 40), (128, 16), (1000, 64)])
def test_select_matches_brute_force(seed, nb, k):
    rng = np.random.default_rng(seed)
    s = rng.standard_normal(nb)
    if seed % 2:  # heavy exact ties
        s = np.round(s * 2) / 2
    sel = oracle.select(s, k)
    want = brute_topk(s.tolist(), k)
    assert sel[: len(want)].tolist() == want
    assert (sel[len(want):] == -1).all()


def test_select_all_permutations_tiny():
    vals = [0.0, 1.0, 1.0, 2.0, 2.0]
    for perm in set(itertools.permutations(vals)):
        for k in range(1, 6):
            assert oracle.select(np.array(perm), k).tolist() == brute_topk(list(perm), k)


def test_select_k1_is_first_argmax_and_ties_go_low():
    s = np.array([1.0, 5.0, 5.0, -2.0])
    assert oracle.select(s, 1).tolist() == [1]
    assert oracle.select(s, 2).tolist() == [1, 2]
    assert oracle.select(np.zeros(9), 4).tolist() == [0, 1, 2, 3]


def test_select_minus_inf_never_beats_finite():
    s = np.array([-np.inf, 0.0, -np.inf, -1e30])
    assert oracle.select(s, 2).tolist() == [1, 3]


def test_select_permutation_equivariance():
    rng = np.random.default_rng(3)
    s = rng.standard_normal(200)   # distinct with probability 1
    perm = rng.permutation(200)
    a = set(oracle.select(s, 20).tolist())
    b = set(oracle.select(s[perm], 20).tolist())
    assert {int(perm[j]) for j in b} == a


def test_split_by_residency():
    sel = np.array([2, 5, 7, 9, -1, -1], dtype=np.int32)
    table = np.full(12, -1, dtype=np.int32)
    table[[2, 9, 10]] = [40, 41, 42]
    sg, ng, sh, nh = oracle.split(sel, table)
    assert (ng, nh) == (2, 2)
    assert sg.tolist() == [2, 9, -1, -1, -1, -1]
    assert sh.tolist() == [5, 7, -1, -1, -1, -1]


# ----------------------------------------------------------------- recall plan


def brute_recall(s, k, table):
    nb = len(s)
    order = sorted(range(nb), key=lambda j: (-s[j], j))
    T = set(order[: min(k, nb)])
    R = {j for j in range(nb) if table[j] >= 0}
    missing = [j for j in order if j in T and j not in R]
    spare = [j for j in order if j in R and j not in T]
    n = min(len(missing), len(spare))
    recall = sorted(missing[:n])
    evict = sorted(spare[len(spare) - n:]) if n else []
    new = list(table)
    slots = [table[e] for e in evict]
    for r, e, sl in zip(recall, evict, slots):
        new[r] = sl
        new[e] = -1
    return recall, slots, evict, new


@pytest.mark.parametrize("seed", range(8))
@pytest.mark.parametrize("nb,k,n_res", [(12, 4, 6), (12, 4, 2), (64, 16, 32), (64, 16, 64), (64, 16, 0), (9, 20, 5)])
def test_recall_plan_matches_brute_force(seed, nb, k, n_res):
    rng = np.random.default_rng(seed)
    s = rng.standard_normal(nb)
    if seed % 3 == 0:
        s = np.round(s * 2) / 2
    table = np.full(nb, -1, dtype=np.int32)
    res = rng.permutation(nb)[:n_res]
    table[res] = rng.permutation(1000)[:n_res]
    want_r, want_s, want_e, want_t = brute_recall(s.tolist(), k, table.tolist())
    t2 = table.copy()
    rb, rs, eb, n = oracle.recall_plan(s, k, t2)
    assert n == len(want_r)
    assert rb[:n].tolist() == want_r and rs[:n].tolist() == want_s and eb[:n].tolist() == want_e
    assert (rb[n:] == -1).all() and (rs[n:] == -1).all() and (eb[n:] == -1).all()
    assert t2.tolist() == want_t
    # invariants: capacity and slot set unchanged, no slot used twice
    assert sorted(t2[t2 >= 0].tolist()) == sorted(table[table >= 0].tolist())
    # when the cache holds at least k blocks the whole top-k is resident afterwards
    if n_res >= min(k, nb):
        T = oracle.select(s, k)
        assert (t2[T[T >= 0]] >= 0).all()
    # a second plan with the same scores moves nothing
    t3 = t2.copy()
    assert oracle.recall_plan(s, k, t3)[3] == 0 or n_res < min(k, nb)
    if n_res >= min(k, nb):
        assert (t3 == t2).all()


# ---------------------------------------------------------------- recall data movement (Sec. 3.4)

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_recall_fetch_is_plain_slicing(dtype):
    rng = np.random.default_rng(41)
    mb, S, d, n_slots = 12, 16, 8, 20
    st = np.float32 if dtype == "f32" else np.uint16
    def arr(shape):
        return W.to_storage(rng.standard_normal(shape).astype(np.float32), dtype)
    src_k, src_v = arr((mb, S, d)), arr((mb, S, d))
    kp, vp = arr((n_slots, S, d)), arr((n_slots, S, d))
    kp0, vp0 = kp.copy(), vp.copy()
    blk = np.array([3, 7, 11, 0, -1, -1], dtype=np.int32)
    slot = np.array([19, 2, 5, 8, -1, -1], dtype=np.int32)
    assert oracle.recall_fetch(src_k, src_v, blk, slot, 4, kp, vp) == 4
    assert kp.dtype == st
    for b, s in zip(blk[:4], slot[:4]):
        assert np.array_equal(kp[s], src_k[b]) and np.array_equal(vp[s], src_v[b])
    rest = [s for s in range(n_slots) if s not in set(slot[:4].tolist())]
    assert np.array_equal(kp[rest], kp0[rest]) and np.array_equal(vp[rest], vp0[rest])
    # K goes to the K pool and V to the V pool, not the other way round
    assert not np.array_equal(kp[19], src_v[3])


def test_recall_fetch_skips_what_is_out_of_range_and_respects_n():
    mb, S, d, n_slots = 4, 2, 2, 3
    src_k = np.arange(mb * S * d, dtype=np.float32).reshape(mb, S, d)
    src_v = -src_k
    kp = np.full((n_slots, S, d), 99.0, dtype=np.float32)
    vp = kp.copy()
    blk = np.array([1, 4, -1, 2, 3], dtype=np.int32)     # 4 and -1 are no blocks
    slot = np.array([0, 1, 1, 3, 2], dtype=np.int32)     # 3 is no slot
    assert oracle.recall_fetch(src_k, src_v, blk, slot, 4, kp, vp) == 1   # entry 4 is beyond n
    assert np.array_equal(kp[0], src_k[1]) and np.array_equal(vp[0], src_v[1])
    assert (kp[1:] == 99.0).all() and (vp[1:] == 99.0).all()


def test_recall_plan_then_fetch_makes_every_selected_block_resident_with_its_own_rows():
    # after plan + transfer, a pool read through the updated table returns the logical block's rows
    rng = np.random.default_rng(43)
    mb, S, d, k = 24, 4, 4, 6
    src_k = rng.standard_normal((mb, S, d)).astype(np.float32)
    src_v = rng.standard_normal((mb, S, d)).astype(np.float32)
    resident = rng.permutation(mb)[:10]
    table = np.full(mb, -1, dtype=np.int32)
    table[resident] = rng.permutation(10).astype(np.int32)
    kp = np.zeros((10, S, d), dtype=np.float32)
    vp = np.zeros((10, S, d), dtype=np.float32)
    kp[table[resident]], vp[table[resident]] = src_k[resident], src_v[resident]
    s = rng.standard_normal(mb)
    rb, rs, eb, n = oracle.recall_plan(s, k, table)
    assert oracle.recall_fetch(src_k, src_v, rb, rs, n, kp, vp) == n
    for j in range(mb):
        if table[j] >= 0:
            assert np.array_equal(kp[table[j]], src_k[j]) and np.array_equal(vp[table[j]], src_v[j])
    top = set(np.argsort(-s, kind="stable")[:k].tolist())
    assert all(table[j] >= 0 for j in top)


# ---------------------------------------------------------------- recall through a staging buffer

def _staged_case(seed, dtype="f32"):
    rng = np.random.default_rng(seed)
    pairs, mb, S, d, k, n_slots = 5, 9, 4, 8, 6, 14
    def arr(shape):
        return W.to_storage(rng.standard_normal(shape).astype(np.float32), dtype)
    src_k, src_v = arr((pairs, mb, S, d)), arr((pairs, mb, S, d))
    n = np.array([3, 0, 6, 1, 9], dtype=np.int32)          # 9 is clamped to k
    blk = np.full((pairs, k), -1, dtype=np.int32)
    slot = np.full((pairs, k), -1, dtype=np.int32)
    free = rng.permutation(n_slots)
    at = 0
    for p in range(pairs):
        m = min(int(n[p]), k)
        blk[p, :m] = rng.permutation(mb)[:m]
        take = min(m, n_slots - at)
        slot[p, :take] = free[at:at + take]
        at += take
    return src_k, src_v, blk, slot, n, arr((n_slots, S, d)), arr((n_slots, S, d)), mb


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_recall_stage_packs_tiles_in_pair_then_entry_order(dtype):
    src_k, src_v, blk, slot, n, kp, vp, mb = _staged_case(51, dtype)
    staged, off = oracle.recall_stage(src_k, src_v, blk, n)
    counts = np.minimum(n, blk.shape[1])
    assert off.tolist() == [0] + np.cumsum(counts)[:-1].tolist()
    assert len(staged) == counts.sum()
    for p in range(len(n)):
        for i in range(counts[p]):
            assert np.array_equal(staged[off[p] + i, 0], src_k[p, blk[p, i]])
            assert np.array_equal(staged[off[p] + i, 1], src_v[p, blk[p, i]])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_recall_stage_then_scatter_is_recall_fetch(dtype):
    src_k, src_v, blk, slot, n, kp, vp, mb = _staged_case(52, dtype)
    # two entries that must be skipped on either route: no such block, no such slot
    blk[2, 1], slot[2, 4] = mb, len(kp)
    kp2, vp2 = kp.copy(), vp.copy()
    moved = sum(oracle.recall_fetch(src_k[p], src_v[p], blk[p], slot[p], min(int(n[p]), blk.shape[1]), kp, vp)
                for p in range(len(n)))
    staged, off = oracle.recall_stage(src_k, src_v, blk, n)
    assert oracle.recall_scatter(staged, off, blk, slot, n, mb, kp2, vp2) == moved
    assert np.array_equal(kp, kp2) and np.array_equal(vp, vp2)
    assert moved == 3 + 0 + 4 + 1 + (slot[4] >= 0).sum()


def test_recall_scatter_reads_the_tile_the_offsets_name():
    # hand-made staging: tile t holds the constant t (K) and -t (V)
    S, d, k, mb = 2, 2, 3, 7
    staged = np.zeros((5, 2, S, d), dtype=np.float32)
    for t in range(5):
        staged[t, 0], staged[t, 1] = t, -t
    off = np.array([0, 2], dtype=np.int32)
    blk = np.array([[4, 6, -1], [0, 1, 2]], dtype=np.int32)
    slot = np.array([[3, 0, -1], [1, 5, 2]], dtype=np.int32)   # 5 is no slot
    n = np.array([2, 3], dtype=np.int32)
    kp = np.full((4, S, d), 99.0, dtype=np.float32)
    vp = kp.copy()
    assert oracle.recall_scatter(staged, off, blk, slot, n, mb, kp, vp) == 4
    assert [kp[s, 0, 0] for s in range(4)] == [1.0, 2.0, 4.0, 0.0]
    assert [vp[s, 0, 0] for s in range(4)] == [-1.0, -2.0, -4.0, -0.0]


# ---------------------------------------------------------------- always-kept blocks

@pytest.mark.parametrize("nb,k,n_sink,n_tail", [(40, 8, 1, 2), (40, 8, 0, 0), (40, 8, 3, 0), (10, 4, 2, 3), (5, 8, 1, 1),
                                                (12, 3, 4, 4), (1, 1, 1, 1), (7, 7, 0, 7)])
def test_forced_blocks_then_topk_is_the_brute_force_rule(nb, k, n_sink, n_tail):
    rng = np.random.default_rng(nb * 100 + k)
    s = rng.standard_normal(nb)
    sel = oracle.select(oracle.force_blocks(s, n_sink, n_tail), k)
    got = [int(j) for j in sel if j >= 0]
    # brute force: forced blocks first in index order, then the others by (score desc, index asc)
    forced = [j for j in range(nb) if j < n_sink or j >= nb - n_tail]
    others = sorted((j for j in range(nb) if j not in forced), key=lambda j: (-s[j], j))
    want = sorted((forced + others)[:min(k, nb)])
    assert got == want
    assert np.array_equal(s, s)   # the input is not modified
    f = oracle.force_blocks(s, n_sink, n_tail)
    assert all(np.isposinf(f[j]) for j in forced) and all(f[j] == s[j] for j in range(nb) if j not in forced)


def test_plan_gap_names_the_only_score_pairs_that_can_change_a_plan():
    """tests/harness.plan_gap is what the GPU parity tests use to excuse a differing plan: scores that
    move by less than a quarter of it (relative) must leave the oracle's plan as it is, and closing
    the deciding gap must be able to change it (so the rule neither hides nor invents mismatches)."""
    from tests import harness
    rng = np.random.default_rng(11)
    changed = 0
    for trial in range(300):
        nb, k = int(rng.integers(4, 60)), int(rng.integers(1, 12))
        s = rng.standard_normal(nb) * 10 + 100
        table = np.where(rng.random(nb) < rng.choice([0.1, 0.5, 0.9]), -1, 0).astype(np.int32)
        table[table >= 0] = rng.permutation(int((table >= 0).sum()))
        g = harness.plan_gap(s, s, k, table)
        t0 = table.copy()
        base = oracle.recall_plan(s, k, t0)
        if not np.isfinite(g):
            continue
        for _ in range(5):
            s2 = s * (1.0 + (rng.random(nb) * 2 - 1) * g / 4)
            t1 = table.copy()
            got = oracle.recall_plan(s2, k, t1)
            assert got[3] == base[3] and all(np.array_equal(a, b) for a, b in zip(got[:3], base[:3])), trial
            assert np.array_equal(t0, t1)
        # noise five times the gap does change some plans
        s3 = s * (1.0 + (rng.random(nb) * 2 - 1) * g * 5)
        t2 = table.copy()
        got = oracle.recall_plan(s3, k, t2)
        changed += int(not all(np.array_equal(a, b) for a, b in zip(got[:3], base[:3])))
    assert changed > 10
