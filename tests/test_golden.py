"""The hand-worked layer-step of tests/golden/hand_worked_layer_step.json: the oracle (CPU) and the
HIP path (GPU) against values derived with pencil and paper from the definitions (Sec. 2.2, Sec. 3.2,
Alg. 1), not from any implementation."""
import json
import math
import os

import numpy as np
import pytest

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))
CASE = json.load(open(os.path.join(HERE, "golden", "hand_worked_layer_step.json")))


def build():
    sh = CASE["shape"]
    d, S, nb = sh["d"], sh["S"], 4
    q = np.zeros((1, 1, d), np.float32)
    q[0, 0, :2] = CASE["q_first_channels"]
    K = np.zeros((nb * S, d), np.float32)
    V = np.zeros((nb * S, d), np.float32)
    for j, kj in enumerate(CASE["block_keys_first_channels"]):
        K[j * S:(j + 1) * S, :2] = kj
    t = np.arange(S, dtype=np.float32)
    V[0 * S:1 * S, :2] = 100.0
    V[2 * S:3 * S, :2] = 100.0
    V[1 * S:2 * S, 0], V[1 * S:2 * S, 1] = t, 1.0
    V[3 * S:4 * S, 0], V[3 * S:4 * S, 1] = -t, 3.0
    table = np.array(CASE["block_table"], np.int32)
    return sh, q, K, V, table


def test_fixture_decimals_agree_with_its_closed_forms():
    e = CASE["expected"]
    r = math.exp(0.0625)
    assert abs(e["out_first_channels_decimal"][0] - 7.5 * math.tanh(0.03125)) < 5e-9
    assert abs(e["out_first_channels_decimal"][1] - (1 + 2 / (1 + r))) < 5e-9
    assert abs(e["lse_decimal"] - (math.log(16) + 0.3125 + math.log(1 + r))) < 5e-9


def test_oracle_reproduces_the_hand_worked_case():
    sh, q, K, V, table = build()
    e = CASE["expected"]
    dig = oracle.digest(K, sh["ctx_len"], sh["S"])
    s = oracle.score(q[0], dig)
    assert s.tolist() == e["scores"]
    s32 = oracle.decision_scores(s)
    assert oracle.select(s32, 2).tolist() == e["sel_all_k2"]
    assert oracle.select(s32, 1).tolist() == e["sel_all_k1"]
    tie = np.array([2.0, 3.0, -1.0, 3.0])
    assert oracle.select(tie, 1).tolist() == [1]                      # the tie goes to the lower index
    sg, ng, shost, nh = oracle.split(oracle.select(s32, 2), table)
    assert sg[:ng].tolist() == e["sel_gpu_k2"] and shost[:nh].tolist() == e["sel_host_k2"]
    og, mg, lg = oracle.partial_attn(q[0, 0], K, V, sg, sh["ctx_len"], sh["S"], sh["sm_scale"])
    oh, mh, lh = oracle.partial_attn(q[0, 0], K, V, shost, sh["ctx_len"], sh["S"], sh["sm_scale"])
    for (o, m, l), want in (((og, mg, lg), e["gpu_partial"]), ((oh, mh, lh), e["host_partial"])):
        assert abs(m - want["m"]) < 1e-12 and abs(l - want["l"]) < 1e-12
        assert np.abs(o[:2] - want["o_first_channels"]).max() < 1e-12 and (o[2:] == 0).all()
    out, lse = oracle.merge(og, mg, lg, oh, mh, lh)
    assert np.abs(out[:2] - e["out_first_channels_decimal"]).max() < 1e-8 and (out[2:] == 0).all()
    assert abs(lse - e["lse_decimal"]) < 1e-8


@pytest.mark.gpu
def test_hip_path_reproduces_the_hand_worked_case():
    import torch

    from paper_2603_27138_amd import binding as B
    sh, q, K, V, table = build()
    e = CASE["expected"]
    d, S, nb = sh["d"], sh["S"], 4
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    ctx = dev(np.array([sh["ctx_len"]], np.int32))
    for k, want_all in ((2, e["sel_all_k2"]), (1, e["sel_all_k1"])):
        p = B.make_problem(1, 1, 1, d, S, B.F32, nb, k, ctx, sh["sm_scale"])
        ws = B.alloc_workspace(p)
        digest = torch.zeros(1, 1, nb, 2, d, device="cuda")
        B.build_digests(p, dev(K.reshape(1, 1, nb, S, d)), digest)
        k_pool = dev(K.reshape(nb, S, d)[[1, 0]])      # slot 0 holds block 1, slot 1 holds block 0
        v_pool = dev(V.reshape(nb, S, d)[[1, 0]])
        # the host's partial, as worked out by hand: only block 3 (k = 2) or nothing (k = 1)
        ho = torch.zeros(1, 1, d, device="cuda")
        hm = torch.full((1, 1), float("-inf"), device="cuda")
        hl = torch.zeros(1, 1, device="cuda")
        if k == 2:
            ho[0, 0, :2] = torch.tensor(e["host_partial"]["o_first_channels"])
            hm[0, 0], hl[0, 0] = e["host_partial"]["m"], e["host_partial"]["l"]
        i32 = dict(dtype=torch.int32, device="cuda")
        scores = torch.empty(1, 1, nb, device="cuda")
        sel_all, sel_gpu, slot_gpu, sel_host = (torch.empty(1, 1, k, **i32) for _ in range(4))
        n_gpu, n_host = torch.empty(1, 1, **i32), torch.empty(1, 1, **i32)
        out, lse = torch.empty(1, 1, d, device="cuda"), torch.empty(1, 1, device="cuda")
        B.layer_step(p, dev(q), digest, dev(table.reshape(1, 1, nb)), k_pool, v_pool, 2, ho, hm, hl, scores, sel_all,
                     sel_gpu, slot_gpu, n_gpu, sel_host, n_host, out, lse, ws)
        assert scores.cpu().numpy().ravel().tolist() == e["scores"]
        assert sel_all.cpu().numpy().ravel().tolist() == want_all
        if k == 2:
            assert sel_gpu.cpu().numpy().ravel().tolist() == [1, -1] and sel_host.cpu().numpy().ravel().tolist() == [3, -1]
            o = out.cpu().numpy().ravel()
            assert np.abs(o[:2] - e["out_first_channels_decimal"]).max() < 1e-5 and (o[2:] == 0).all()
            assert abs(float(lse) - e["lse_decimal"]) < 1e-5
        else:
            o = out.cpu().numpy().ravel()
            assert np.abs(o[:2] - e["gpu_partial"]["o_first_channels"]).max() < 1e-5
            assert abs(float(lse) - (0.375 + math.log(16))) < 1e-5
