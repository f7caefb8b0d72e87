"""The whole re-layout pipeline of the paper on one GPU: N ranks' buffers side by side, every stage through
the C ABI, the All-to-Alls replaced by row copies between the ranks' buffers (torch slicing, test-side glue):

    gate (per rank) -> routing counts R -> planner (expert layout, host C++) -> FSEP unshard of the hosted
    experts -> token dispatcher (lite routing + permutation, per rank) -> [exchange] -> grouped FFN on every
    device over its own C slots -> [exchange back] -> combine (per rank);
    backward: combine bwd -> [exchange] -> grouped FFN bwd per device -> [exchange back] -> permute bwd,
    gate bwd; weight gradients of the slots -> FSEP reshard (sum over replicas).

Each rank's output must equal, bit for bit, what the plain single-device path computes for that rank's
tokens (re-layout changes where rows are computed, not their arithmetic: section 3.1, "numerical precision
identical"), and everything must sit within the bf16 bar of the dense oracle; the resharded weight
gradients must match the oracle's gradients summed over ranks."""
import numpy as np
import pytest
import torch

from oracle import oracle as O
from paper_2602_11686_amd import binding as B
from paper_2602_11686_amd import fsep as F
from paper_2602_11686_amd import inputs as I
from paper_2602_11686_amd import planner as P
from tests.gpu_common import TOL, host
from tests.helpers import rel_max

pytestmark = pytest.mark.gpu

BF = torch.bfloat16


def bits(rng, shape, std=1.0):
    return I.f32_to_bf16_bits((rng.standard_normal(shape) * std).astype(np.float32))


def to_gpu(b):
    return torch.tensor(b.view(np.int16), device="cuda").view(BF)


def f64(b):
    return I.bf16_bits_to_f32(b).astype(np.float64)


def i32(a):
    return torch.tensor(np.asarray(a, dtype=np.int32), dtype=torch.int32, device="cuda")


@pytest.mark.parametrize("N,D,E,C,k,T,d,f", [(4, 2, 6, 2, 2, 192, 128, 192), (8, 4, 8, 2, 2, 96, 64, 128)])
def test_relayout_pipeline_equals_the_single_device_layer(N, D, E, C, k, T, d, f):
    print(f"case N={N} D={D} E={E} C={C} k={k} T={T} d={d} f={f}", flush=True)
    rng = np.random.default_rng(N * 10 + E)
    wg_b, w1_b, w3_b, w2_b = bits(rng, (d, E), 0.3), bits(rng, (E, d, f), 0.05), bits(rng, (E, d, f), 0.05), bits(rng, (E, f, d), 0.05)
    skew = np.linspace(1.5, -1.5, E).astype(np.float32)                     # a skewed gate: the early experts are hot
    x_b = [bits(rng, (T, d)) for _ in range(N)]
    dy_b = [bits(rng, (T, d)) for _ in range(N)]
    wg, w1, w3, w2 = to_gpu(wg_b), to_gpu(w1_b), to_gpu(w3_b), to_gpu(w2_b)
    bias = torch.tensor(skew, device="cuda")
    s = B.Shape(T, d, f, E, k, BF)
    ws = torch.empty(B.moe_workspace_bytes(s), dtype=torch.uint8, device="cuda")
    R_rows = T * k
    psi = 3 * d * f

    # ---- every rank: gate; routing counts -> planner --------------------------------------------------
    x = [to_gpu(b) for b in x_b]
    dy = [to_gpu(b) for b in dy_b]
    ids = [torch.empty(T, k, dtype=torch.int32, device="cuda") for _ in range(N)]
    tw = [torch.empty(T, k, dtype=torch.float32, device="cuda") for _ in range(N)]
    for i in range(N):
        B.moe_gate_topk(s, x[i], wg, bias, ids[i], tw[i], None, ws)
    torch.cuda.synchronize()
    Rm = np.stack([np.bincount(host(ids[i]).reshape(-1), minlength=E) for i in range(N)]).astype(np.int64)
    ps = P.PlanShape(N, E, C, D)
    cost = P.PlanCost(v_comm=2.0 * d, b_intra=64e9, b_inter=25e9, v_comp=6.0 * d * f, b_comp=1e15, f_ckpt=0)
    A, _, _ = P.moe_plan_expert_layout(ps, cost, Rm, 4, 1)
    assert (A.sum(axis=1) == C).all()
    hosted = np.stack([np.repeat(np.arange(E), A[i]) for i in range(N)]).astype(np.int32)      # slot order = group order
    assert (Rm.sum(axis=0) > 0).any() and A.max() >= 1

    # ---- FSEP: shard the experts, restore the hosted ones on every device ------------------------------
    flat = torch.cat([w1.reshape(E, -1), w3.reshape(E, -1), w2.reshape(E, -1)], dim=1).contiguous()
    shards = torch.empty(N, E, psi // N, dtype=BF, device="cuda")
    restored = torch.empty(N, C, psi, dtype=BF, device="cuda")
    F.moe_fsep_shard(N, flat, shards)
    F.moe_fsep_unshard(shards, i32(hosted), restored)
    w1_loc = [restored[kdev, :, :d * f].reshape(C, d, f).contiguous() for kdev in range(N)]
    w3_loc = [restored[kdev, :, d * f:2 * d * f].reshape(C, d, f).contiguous() for kdev in range(N)]
    w2_loc = [restored[kdev, :, 2 * d * f:].reshape(C, f, d).contiguous() for kdev in range(N)]

    # ---- every rank: token dispatcher -------------------------------------------------------------------
    G = N * C
    disp = []
    for i in range(N):
        Gi, eog, dog, rb, rg = P.moe_plan_dispatch_table(ps, A, i)
        assert Gi == G and (eog == hosted.reshape(-1)).all()
        ec = torch.empty(E, dtype=torch.int32, device="cuda"); gc = torch.empty(G, dtype=torch.int32, device="cuda")
        go = torch.empty(G + 1, dtype=torch.int32, device="cuda")
        rop = torch.empty(R_rows, dtype=torch.int32, device="cuda"); por = torch.empty_like(rop)
        xp = torch.empty(R_rows, d, dtype=BF, device="cuda"); err = torch.zeros(1, dtype=torch.int32, device="cuda")
        B.moe_permute_lite(s, G, x[i], ids[i], i32(rb), i32(rg), ec, gc, go, rop, por, xp, err, ws)
        torch.cuda.synchronize()
        assert int(err[0]) == 0
        disp.append(dict(go=host(go), rop=rop, xp=xp))

    # ---- exchange: device kdev receives, slot by slot, the rows every rank holds for its groups ---------
    def gather(per_rank_rows):
        recv, offs, book = [], [], []
        for kdev in range(N):
            parts, off, bk = [], [0], []
            for c in range(C):
                g = kdev * C + c
                for i in range(N):
                    a, b = int(disp[i]["go"][g]), int(disp[i]["go"][g + 1])
                    if b > a:
                        parts.append(per_rank_rows[i][a:b])
                        bk.append((i, a, b))
                off.append(off[-1] + sum(int(disp[i]["go"][g + 1] - disp[i]["go"][g]) for i in range(N)))
            recv.append(torch.cat(parts) if parts else torch.empty(0, per_rank_rows[0].shape[1], dtype=BF, device="cuda"))
            offs.append(off)
            book.append(bk)
        return recv, offs, book

    def scatter_back(per_dev_rows, book, width):
        out = [torch.empty(R_rows, width, dtype=BF, device="cuda") for _ in range(N)]
        for kdev in range(N):
            pos = 0
            for (i, a, b) in book[kdev]:
                out[i][a:b] = per_dev_rows[kdev][pos:pos + (b - a)]
                pos += b - a
        return out

    recv, offs, book = gather([disp[i]["xp"] for i in range(N)])
    dev_state = []
    for kdev in range(N):
        Rk = recv[kdev].shape[0]
        if Rk == 0:
            dev_state.append(None)
            continue
        sk = B.Shape(Rk, d, f, C, 1, BF)
        wsk = torch.empty(B.moe_workspace_bytes(sk), dtype=torch.uint8, device="cuda")
        yp = torch.empty(Rk, d, dtype=BF, device="cuda")
        a_s = torch.empty(Rk, f, dtype=BF, device="cuda"); b_s = torch.empty_like(a_s)
        B.moe_grouped_ffn_fwd(sk, recv[kdev], i32(offs[kdev]), w1_loc[kdev], w3_loc[kdev], w2_loc[kdev], yp, a_s, b_s, wsk)
        dev_state.append(dict(sk=sk, ws=wsk, yp=yp, a=a_s, b=b_s, off=i32(offs[kdev])))
    yp_rank = scatter_back([st["yp"] if st else torch.empty(0, d, dtype=BF, device="cuda") for st in dev_state], book, d)
    y = [torch.empty(T, d, dtype=BF, device="cuda") for _ in range(N)]
    for i in range(N):
        B.moe_unpermute_combine(s, yp_rank[i], disp[i]["rop"], tw[i], y[i])

    # ---- backward ------------------------------------------------------------------------------------------
    dyp_rank, dtw = [], []
    for i in range(N):
        dyp = torch.empty(R_rows, d, dtype=BF, device="cuda"); dw_i = torch.empty(T, k, dtype=torch.float32, device="cuda")
        B.moe_combine_bwd(s, dy[i], yp_rank[i], disp[i]["rop"], tw[i], dyp, dw_i)
        dyp_rank.append(dyp); dtw.append(dw_i)
    drecv, _, _ = gather(dyp_rank)
    grads = torch.zeros(N, C, psi, dtype=BF, device="cuda")
    dxp_dev = []
    for kdev in range(N):
        st = dev_state[kdev]
        if st is None:
            dxp_dev.append(torch.empty(0, d, dtype=BF, device="cuda"))
            continue
        Rk = recv[kdev].shape[0]
        dxp = torch.empty(Rk, d, dtype=BF, device="cuda")
        dw1 = torch.empty(C, d, f, dtype=BF, device="cuda"); dw3 = torch.empty_like(dw1); dw2 = torch.empty(C, f, d, dtype=BF, device="cuda")
        B.moe_grouped_ffn_bwd(st["sk"], recv[kdev], st["off"], w1_loc[kdev], w3_loc[kdev], w2_loc[kdev], st["a"], st["b"],
                              drecv[kdev], dxp, dw1, dw3, dw2, st["ws"])
        grads[kdev] = torch.cat([dw1.reshape(C, -1), dw3.reshape(C, -1), dw2.reshape(C, -1)], dim=1)
        dxp_dev.append(dxp)
    dxp_rank = scatter_back(dxp_dev, book, d)
    dx = [torch.empty(T, d, dtype=BF, device="cuda") for _ in range(N)]
    dwg = [torch.empty(d, E, dtype=torch.float32, device="cuda") for _ in range(N)]
    for i in range(N):
        B.moe_unpermute_combine(s, dxp_rank[i], disp[i]["rop"], None, dx[i])
        B.moe_gate_topk_bwd(s, x[i], wg, ids[i], tw[i], dtw[i], dx[i], dwg[i], ws)
    gsh = torch.empty(N, E, psi // N, dtype=BF, device="cuda")
    F.moe_fsep_reshard(grads, i32(hosted), gsh)
    torch.cuda.synchronize()
    gflat = gsh.permute(1, 0, 2).reshape(E, psi)
    dW1 = host(gflat[:, :d * f]).reshape(E, d, f); dW3 = host(gflat[:, d * f:2 * d * f]).reshape(E, d, f)
    dW2 = host(gflat[:, 2 * d * f:]).reshape(E, f, d)

    # ---- the plain single-device path on every rank's tokens: identical bits ---------------------------
    for i in range(N):
        counts = torch.empty(E, dtype=torch.int32, device="cuda"); offsets = torch.empty(E + 1, dtype=torch.int32, device="cuda")
        rop = torch.empty(R_rows, dtype=torch.int32, device="cuda"); por = torch.empty_like(rop)
        xp = torch.empty(R_rows, d, dtype=BF, device="cuda"); yp = torch.empty_like(xp); y_plain = torch.empty(T, d, dtype=BF, device="cuda")
        B.moe_permute(s, x[i], ids[i], counts, offsets, rop, por, xp, ws)
        B.moe_grouped_ffn_fwd(s, xp, offsets, w1, w3, w2, yp, None, None, ws)
        B.moe_unpermute_combine(s, yp, rop, tw[i], y_plain)
        torch.cuda.synchronize()
        assert torch.equal(y[i].view(torch.int16), y_plain.view(torch.int16)), f"rank {i}"

    # ---- the dense oracle ----------------------------------------------------------------------------------
    Wg, W1, W3, W2 = f64(wg_b), f64(w1_b), f64(w3_b), f64(w2_b)
    tot1, tot3, tot2 = np.zeros_like(W1), np.zeros_like(W3), np.zeros_like(W2)
    for i in range(N):
        fw = O.layer_fwd(f64(x_b[i]), Wg, skew.astype(np.float64), W1, W3, W2, k)
        np.testing.assert_array_equal(host(ids[i]), fw["ids"])
        bw = O.layer_bwd(f64(x_b[i]), Wg, W1, W3, W2, fw, f64(dy_b[i]))
        assert rel_max(host(y[i]), fw["Y"]) <= TOL[BF]
        assert rel_max(host(dx[i]), bw["dX"]) <= TOL[BF]
        assert rel_max(host(dwg[i]), bw["dWg"]) <= TOL[BF]
        tot1 += bw["dW1"]; tot3 += bw["dW3"]; tot2 += bw["dW2"]
    assert rel_max(dW1, tot1) <= TOL[BF] and rel_max(dW3, tot3) <= TOL[BF] and rel_max(dW2, tot2) <= TOL[BF]
