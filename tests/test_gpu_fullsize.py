"""GPU parity at the FULL sizes of the benchmark workloads, in the launch configuration bench.py
times.  The fp64 oracle cannot finish these shapes, so it is evaluated on sampled outputs:

  * forward: sampled query rows of sampled (b, h) -- a row of O / LSE depends on nothing else;
  * dQ:      the same rows -- a row of dQ depends only on that row's scores;
  * dK, dV:  sampled key columns.  Their gradients sum over every query row whose mask admits
             them; those rows are found by evaluating the ORACLE's mask_mod on the whole
             (rows x sampled columns) grid, and the oracle's backward is run on exactly those rows
             for every query head of the group.

Tolerances are those of test_gpu_parity.py.
"""
import pytest
import torch

import flex_workloads as wlm
from oracle import flex_oracle as fo

from helpers import check_grad, check_output, oracle_mods, run_backward, run_forward

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def rows_seeing(mask_mod, b, h, S, cols):
    keep = mask_mod(b, h, torch.arange(S).view(-1, 1), cols.view(1, -1))
    return torch.nonzero(keep.expand(S, cols.numel()).any(dim=1)).flatten()


def check_full_size(wl, heads, n_rows, col_groups):
    inp = wlm.make_train_inputs(wl, with_dO=True)
    score, mask = oracle_mods(wl, inp)
    print(f"[case] {wl.name}: forward + backward on the GPU", flush=True)
    O, LSE, bm, ids = run_forward(wl, inp, DEV)
    dQ, dK, dV = run_backward(wl, inp, DEV, O, LSE, bm, ids)
    # the backward that keeps dS in memory: dK / dV come from the same kernel (same bits), its dQ is
    # checked on the sampled rows like the other one
    dQ_st, dK_st, dV_st = run_backward(wl, inp, DEV, O, LSE, bm, ids, stored=True)
    assert torch.equal(dK_st, dK) and torch.equal(dV_st, dV)
    del dK_st, dV_st
    O, LSE, dQ, dK, dV, dQ_st = (t.cpu() for t in (O, LSE, dQ, dK, dV, dQ_st))
    G = wl.Hq // wl.Hkv
    gen = torch.Generator().manual_seed(wl.seed + 7)
    for (b, h) in heads:
        rows = torch.randint(0, wl.S, (n_rows,), generator=gen)
        rows = torch.unique(torch.cat([rows, torch.tensor([0, 1, wl.Bq - 1, wl.Bq, wl.S - 1])]))
        print(f"[case] {wl.name}: rows of (b={b}, h={h})", flush=True)
        args = (inp.Q[b, h], inp.K[b, h // G], inp.V[b, h // G])
        o_ref, l_ref = fo.attention_head(*args, score, mask, inp.scale, b, h, q_rows=rows)
        check_output(O[b, h, rows], LSE[b, h, rows], o_ref, l_ref)
        dq_ref, _, _ = fo.attention_head_backward(*args, inp.dO[b, h], score, mask, inp.scale, b, h, q_rows=rows)
        check_grad("dQ", dQ[b, h, rows], dq_ref)
        check_grad("dQ (dS kept in memory)", dQ_st[b, h, rows], dq_ref)
    for (b, hkv, cols) in col_groups:
        dk_ref = torch.zeros(cols.numel(), wl.D, dtype=torch.float64)
        dv_ref = torch.zeros_like(dk_ref)
        for g in range(G):
            h = hkv * G + g
            rows = rows_seeing(mask, b, h, wl.S, cols)
            print(f"[case] {wl.name}: dK/dV of (b={b}, hkv={hkv}) cols {int(cols[0])}..{int(cols[-1])}: "
                  f"head {h}, {rows.numel()} rows", flush=True)
            if rows.numel() == 0:
                continue
            _, dk, dv = fo.attention_head_backward(inp.Q[b, h], inp.K[b, hkv], inp.V[b, hkv], inp.dO[b, h], score,
                                                   mask, inp.scale, b, h, q_rows=rows, stripe=512)
            dk_ref += dk[cols]
            dv_ref += dv[cols]
        check_grad("dK", dK[b, hkv, cols], dk_ref)
        check_grad("dV", dV[b, hkv, cols], dv_ref)


def test_cfg2_dense_causal_softcap_full_size():
    wl = wlm.CFG2
    check_full_size(wl, heads=[(0, 0), (1, 7), (3, 15)], n_rows=40,
                    col_groups=[(0, 0, torch.arange(wl.S - 128, wl.S)), (2, 5, torch.arange(6000, 6064)),
                                (3, 15, torch.arange(8000, 8020))])


def test_cfg3_document_alibi_full_size():
    wl = wlm.CFG3
    check_full_size(wl, heads=[(0, 0), (0, 9), (0, 15)], n_rows=40,
                    col_groups=[(0, 3, torch.arange(wl.S - 64, wl.S)), (0, 12, torch.arange(5000, 5064))])


def test_cfg4_swa_prefix_relbias_gqa_full_size():
    wl = wlm.CFG4
    check_full_size(wl, heads=[(0, 0), (1, 13), (1, 31)], n_rows=24,
                    col_groups=[(0, 2, torch.arange(wl.S - 96, wl.S)), (1, 7, torch.arange(20000, 20032)),
                                (0, 0, torch.arange(1024, 1032))])

