"""Pins for the oracle's decode append (CPU only).

The digest is the one of Sec. 2.2 (channel-wise min/max over a block's keys): whatever order the
keys arrive in, the digest and the tiles after n appends must be those of the finished sequence.
The checks below use numpy min/max and plain slicing, not the oracle's own digest routine, and a
second group cross-checks against that routine as well.
"""
import numpy as np
import pytest

import oracle
from paper_2603_27138_amd import workload as W


def _rand(shape, seed, dtype):
    x = np.random.default_rng(seed).standard_normal(shape).astype(np.float32)
    return W.to_storage(x, dtype)


def _run(dtype, S, d, max_blocks, n, seed, host_every=3, start=0, K0=None, V0=None):
    """Append tokens start..n-1 one by one.  Blocks j with j % host_every == host_every-1 go to the host."""
    code = oracle.F32 if dtype == "f32" else oracle.BF16
    K = _rand((n, d), seed, dtype) if K0 is None else K0
    V = _rand((n, d), seed + 1, dtype) if V0 is None else V0
    dig = np.zeros((max_blocks, 2, d), dtype=K.dtype)
    table = np.full(max_blocks, -7, dtype=np.int32)
    n_slots = max_blocks
    kp = np.zeros((n_slots, S, d), dtype=K.dtype)
    vp = np.zeros((n_slots, S, d), dtype=K.dtype)
    ctx = start
    free = list(range(n_slots))[::-1]
    for t in range(start, n):
        new_slot = -1
        if t % S == 0:
            new_slot = -1 if (t // S) % host_every == host_every - 1 else free.pop()
        ctx2 = oracle.append(code, S, ctx, K[t].copy(), V[t].copy(), new_slot, dig, table, kp, vp)
        assert ctx2 == ctx + 1
        ctx = ctx2
    return K, V, dig, table, kp, vp, ctx


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("S,d,n", [(16, 8, 100), (32, 64, 65), (16, 128, 16), (64, 4, 1)])
def test_append_gives_minmax_of_the_finished_blocks(dtype, S, d, n):
    max_blocks = (n + S - 1) // S + 2
    K, V, dig, table, kp, vp, ctx = _run(dtype, S, d, max_blocks, n, seed=11)
    assert ctx == n
    nb = (n + S - 1) // S
    Kf = W.storage_to_f32(K).astype(np.float64)
    df = W.storage_to_f32(dig).astype(np.float64)
    for j in range(nb):
        blk = Kf[j * S:min(n, (j + 1) * S)]
        assert np.array_equal(df[j, 0], blk.min(axis=0))
        assert np.array_equal(df[j, 1], blk.max(axis=0))
    # bit for bit the same as the digest of the whole sequence built in one piece
    assert np.array_equal(dig[:nb], oracle.digest(K, n, S))
    # blocks never opened are untouched
    assert (dig[nb:] == 0).all() and (table[nb:] == -7).all()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_append_fills_tiles_of_resident_blocks_only(dtype):
    S, d, n = 16, 8, 75
    K, V, dig, table, kp, vp, ctx = _run(dtype, S, d, 8, n, seed=5, host_every=2)
    nb = (n + S - 1) // S
    used = set()
    for j in range(nb):
        t0, t1 = j * S, min(n, (j + 1) * S)
        if j % 2 == 1:
            assert table[j] == -1
            continue
        s = table[j]
        assert 0 <= s < len(kp) and s not in used
        used.add(s)
        assert np.array_equal(kp[s, :t1 - t0], K[t0:t1]) and np.array_equal(vp[s, :t1 - t0], V[t0:t1])
        assert (kp[s, t1 - t0:] == 0).all() and (vp[s, t1 - t0:] == 0).all()
    for s in range(len(kp)):
        if s not in used:
            assert (kp[s] == 0).all() and (vp[s] == 0).all()


def test_append_keeps_the_older_of_equal_keys_and_signed_zeros():
    # ties keep the element already stored, so -0.0 and +0.0 stay as first seen: same rule as a
    # first-occurrence min/max over the block
    S, d = 4, 2
    K = np.array([[0.0, -0.0], [-0.0, 0.0], [0.0, 0.0], [1.0, -1.0]], dtype=np.float32)
    V = np.zeros_like(K)
    _, _, dig, _, _, _, _ = _run("f32", S, d, 2, 4, seed=0, K0=K, V0=V)
    assert np.array_equal(np.signbit(dig[0, 0]), [False, True])   # min row: first-seen zero, then -1
    assert np.array_equal(dig[0, 0], np.array([0.0, -1.0], dtype=np.float32))
    assert np.array_equal(np.signbit(dig[0, 1]), [False, True])   # max row: 1, and the first-seen -0.0
    assert np.array_equal(dig[0, 1], np.array([1.0, -0.0], dtype=np.float32))


def test_append_on_a_full_sequence_changes_nothing():
    S, d, mb = 4, 4, 2
    K, V, dig, table, kp, vp, ctx = _run("f32", S, d, mb, mb * S, seed=3, host_every=100)
    before = [a.copy() for a in (dig, table, kp, vp)]
    k = np.full(d, 100.0, dtype=np.float32)
    assert oracle.append(oracle.F32, S, ctx, k, k.copy(), 0, dig, table, kp, vp) == ctx
    for a, b in zip(before, (dig, table, kp, vp)):
        assert np.array_equal(a, b)


def test_append_a_planted_mistake_would_show():
    # an update that compared against the wrong row (max against the min row) or that skipped the
    # r == 0 reset must fail the min/max pin: emulate both on a copy and check they differ
    S, d, n = 8, 4, 20
    K, V, dig, *_ = _run("f32", S, d, 4, n, seed=9)
    Kf = K.astype(np.float64)
    no_reset_min = np.minimum.accumulate(Kf, axis=0)[n - 1]          # never reset at block starts
    assert not np.array_equal(dig[2, 0].astype(np.float64), no_reset_min)
    swapped = Kf[16:20].max(axis=0)
    assert not np.array_equal(dig[2, 0].astype(np.float64), swapped)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_append_keeps_the_host_copy_complete(dtype):
    # with a host copy, every token lands there whatever the block's residency: afterwards the copy is
    # the sequence itself, block by block
    S, d, n, mb = 8, 4, 29, 5
    code = oracle.F32 if dtype == "f32" else oracle.BF16
    K, V = _rand((n, d), 31, dtype), _rand((n, d), 32, dtype)
    dig = np.zeros((mb, 2, d), dtype=K.dtype)
    table = np.full(mb, -7, dtype=np.int32)
    kp, vp = np.zeros((mb, S, d), dtype=K.dtype), np.zeros((mb, S, d), dtype=K.dtype)
    hk, hv = np.zeros((mb, S, d), dtype=K.dtype), np.zeros((mb, S, d), dtype=K.dtype)
    ctx, free = 0, [4, 2, 0]
    for t in range(n):
        slot = (free.pop() if (t // S) % 2 == 0 else -1) if t % S == 0 else -9
        ctx = oracle.append(code, S, ctx, K[t].copy(), V[t].copy(), slot, dig, table, kp, vp, hk, hv)
    assert ctx == n
    flat_k, flat_v = hk.reshape(mb * S, d), hv.reshape(mb * S, d)
    assert np.array_equal(flat_k[:n], K) and np.array_equal(flat_v[:n], V)
    assert (flat_k[n:] == 0).all() and (flat_v[n:] == 0).all()
    # and a resident block's tile holds the same rows as the host copy
    for j in range((n + S - 1) // S):
        if table[j] >= 0:
            rows = min(S, n - j * S)
            assert np.array_equal(kp[table[j], :rows], hk[j, :rows]) and np.array_equal(vp[table[j], :rows], hv[j, :rows])
