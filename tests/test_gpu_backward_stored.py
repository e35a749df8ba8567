"""GPU parity of flexattn_backward_stored -- the backward that writes dS to memory in the dK/dV kernel
and computes dQ = scale * dS K from what was written -- against the fp64 oracle, on the cases of
test_gpu_parity.py (every block-size pair, GQA, per-batch and per-head BlockMasks, compositions),
ragged lengths, and a column walk of more than one list segment.  dK and dV come from the same kernel
as in flexattn_backward and must have the same bits; dQ is held to the same tolerance as there.
(The full-size configurations are covered in test_gpu_fullsize.py.)
"""
import pytest
import torch

import flex_workloads as wlm
from oracle import flex_oracle as fo

from helpers import (check_grad, emulate_bf16_backward, library_mods, nonempty_blocks, oracle_mods, run_backward,
                     run_forward)
from test_gpu_parity import PER_HEAD, SMALL

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def check_case(wl, Hm=1):
    inp = wlm.make_train_inputs(wl, with_dO=True)
    score, mask = oracle_mods(wl, inp)
    O, LSE, bm, ids = run_forward(wl, inp, DEV, Hm=Hm)
    dQ, dK, dV = run_backward(wl, inp, DEV, O, LSE, bm, ids, stored=True)
    g_ref = fo.flex_attention_backward(inp.Q, inp.K, inp.V, inp.dO, score, mask, inp.scale)
    g_em = emulate_bf16_backward(inp, score, mask)
    for n, g, r, e in zip(("dQ", "dK", "dV"), (dQ, dK, dV), g_ref, g_em):
        check_grad(n, g, r, e)
    dQ1, dK1, dV1 = run_backward(wl, inp, DEV, O, LSE, bm, ids)
    assert torch.equal(dK, dK1) and torch.equal(dV, dV1)
    # the two dQ sum the same bf16 dS in different orders (fp32 accumulation): a few bf16 ulps apart
    diff = (dQ.float() - dQ1.float()).abs().max().item()
    assert diff <= 2e-2 * max(1.0, g_ref[0].abs().max().item()), diff
    # twice the same bits (no atomics)
    dQ2, _, _ = run_backward(wl, inp, DEV, O, LSE, bm, ids, stored=True)
    assert torch.equal(dQ, dQ2)


@pytest.mark.parametrize("name", list(SMALL))
def test_stored_small(name):
    wl = SMALL[name]
    if not wl.backward:
        pytest.skip("forward-only configuration")
    print(f"[case] dS kept in memory: {name} {wl}", flush=True)
    check_case(wl)


@pytest.mark.parametrize("name", list(PER_HEAD))
def test_stored_per_head_blockmask(name):
    wl = PER_HEAD[name]
    print(f"[case] dS kept in memory, per-head BlockMask: {name} {wl}", flush=True)
    check_case(wl, Hm=wl.Hq)


RAGGED = [
    ("causal_softcap_d128_s1000", wlm.CFG2, dict(B=1, Hq=2, Hkv=2, S=1000), None),
    ("none_d64_300x777_bk128", wlm.CFG1, dict(B=1, Hq=2, Hkv=1, S=777, D=64, Bq=64, Bk=128, mask="none", backward=True), 300),
    ("causal_d64_q1_kv65", wlm.CFG1, dict(B=2, Hq=2, Hkv=2, S=65, backward=True), 1),
    ("swa_prefix_relbias_gqa_d128_s999", wlm.CFG4, dict(B=1, Hq=4, Hkv=2, S=999, window=200, prefix_len=100, rel_len=64), None),
    ("none_d128_s130_bk128", wlm.CFG2, dict(B=1, Hq=1, Hkv=1, S=130, Bq=64, Bk=128, mask="none", score="identity"), None),
]


@pytest.mark.parametrize("case", RAGGED, ids=[c[0] for c in RAGGED])
def test_stored_ragged_lengths(case):
    """Lengths that are no multiple of the block size (and, with Bk = 128, a last block whose second
    half lies wholly past kv_len, for which no dS is ever written); guard rows behind dQ."""
    import paper_2412_05496_amd as fa
    name, base, over, q_len = case
    wl = base.scaled(name="stored_ragged_" + name, seed=4500 + len(name), **over)
    inp = wlm.make_train_inputs(wl, with_dO=True)
    Lq = wl.S if q_len is None else q_len
    Q, dO = inp.Q[:, :, :Lq].contiguous(), inp.dO[:, :, :Lq].contiguous()
    score_mod, mask_mod = oracle_mods(wl, inp)
    dQ_ref, dK_ref, dV_ref = fo.flex_attention_backward(Q, inp.K, inp.V, dO, score_mod, mask_mod, inp.scale)
    print(f"[case] dS kept in memory, ragged: {name} {wl} q_len {Lq}", flush=True)

    mask_id, score_id, params, Bm = library_mods(wl, inp, DEV)
    bm = fa.alloc_blockmask(Bm, 1, Lq, wl.S, wl.Bq, wl.Bk, device=DEV)
    fa.flexattn_blockmask_build(mask_id, params, bm)
    Qd, Kd, Vd, dOd = Q.to(DEV), inp.K.to(DEV), inp.V.to(DEV), dO.to(DEV)
    O = torch.empty_like(Qd)
    LSE = torch.empty(Qd.shape[:3], dtype=torch.float32, device=DEV)
    fa.flexattn_forward(Qd, Kd, Vd, score_id, mask_id, params, bm, inp.scale, O, LSE)
    dQ_buf = torch.full((Qd.shape[0], Qd.shape[1], Lq + 64, Qd.shape[3]), 7.0, dtype=Qd.dtype, device=DEV)
    dQ = dQ_buf[:, :, :Lq]
    dK, dV = torch.empty_like(Kd), torch.empty_like(Vd)
    n_blocks = nonempty_blocks(bm)
    # a workspace full of NaN bit patterns: whatever is read without having been written shows up
    ws = torch.full((fa.flexattn_backward_stored_workspace_bytes(Qd, Kd, bm, n_blocks),), 0xFF, dtype=torch.uint8,
                    device=DEV)
    fa.flexattn_backward_stored(Qd, Kd, Vd, O, dOd, LSE, score_id, mask_id, params, bm, inp.scale, dQ, dK, dV,
                                n_blocks, ws)
    torch.cuda.synchronize()
    check_grad("dQ", dQ, dQ_ref)
    check_grad("dK", dK, dK_ref)
    check_grad("dV", dV, dV_ref)
    assert (dQ_buf[:, :, Lq:] == 7.0).all()


def test_stored_walk_longer_than_one_segment():
    """A row of blocks with more tiles than one list segment of the dQ kernel holds (512), and key
    columns whose walk in the dK/dV kernel has more than one segment as well: 66 560 keys, 66 560 query
    rows would be too much for the oracle, so q_len = 128 against kv_len = 66 560 (no mask) covers the
    first, and q_len = 66 560 against kv_len = 128 the second."""
    import paper_2412_05496_amd as fa
    for (Lq, Lk) in ((128, 66560), (66560, 128)):
        wl = wlm.Workload("stored_long", B=1, Hq=1, Hkv=1, S=max(Lq, Lk), D=64, Bq=64, Bk=64, mask="none",
                          score="identity", seed=77)
        inp = wlm.make_train_inputs(wl, with_dO=True)
        Q, dO = inp.Q[:, :, :Lq].contiguous(), inp.dO[:, :, :Lq].contiguous()
        K, V = inp.K[:, :, :Lk].contiguous(), inp.V[:, :, :Lk].contiguous()
        score_mod, mask_mod = oracle_mods(wl, inp)
        print(f"[case] dS kept in memory, long walk: q_len {Lq} kv_len {Lk}", flush=True)
        dQ_ref, dK_ref, dV_ref = fo.flex_attention_backward(Q, K, V, dO, score_mod, mask_mod, inp.scale)
        mask_id, score_id, params, Bm = library_mods(wl, inp, DEV)
        bm = fa.alloc_blockmask(1, 1, Lq, Lk, 64, 64, device=DEV)
        fa.flexattn_blockmask_build(mask_id, params, bm)
        Qd, Kd, Vd, dOd = Q.to(DEV), K.to(DEV), V.to(DEV), dO.to(DEV)
        O = torch.empty_like(Qd)
        LSE = torch.empty(Qd.shape[:3], dtype=torch.float32, device=DEV)
        fa.flexattn_forward(Qd, Kd, Vd, score_id, mask_id, params, bm, inp.scale, O, LSE)
        dQ, dK, dV = torch.empty_like(Qd), torch.empty_like(Kd), torch.empty_like(Vd)
        fa.flexattn_backward_stored(Qd, Kd, Vd, O, dOd, LSE, score_id, mask_id, params, bm, inp.scale, dQ, dK, dV,
                                    nonempty_blocks(bm))
        torch.cuda.synchronize()
        check_grad("dQ", dQ, dQ_ref)
        check_grad("dK", dK, dK_ref)
        check_grad("dV", dV, dV_ref)


def test_stored_capacity_and_workspace_errors():
    """Too small a workspace is an error; too small a CAPACITY is the caller's mistake and gives wrong
    numbers, but every slot is clamped: the call returns and what it wrote is finite."""
    import paper_2412_05496_amd as fa
    wl = SMALL["cfg2_small"]
    inp = wlm.make_train_inputs(wl, with_dO=True)
    O, LSE, bm, ids = run_forward(wl, inp, DEV)
    mask_id, score_id, params, Q, K, V = ids
    dO = inp.dO.to(DEV)
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)
    n_blocks = nonempty_blocks(bm)
    need = fa.flexattn_backward_stored_workspace_bytes(Q, K, bm, n_blocks)
    assert need > n_blocks * wl.Bq * wl.Bk * 2 * wl.B * wl.Hq
    assert fa.flexattn_backward_stored_workspace_bytes(Q, K, bm, -1) == 0
    args = (Q, K, V, O, dO, LSE, score_id, mask_id, params, bm, inp.scale, dQ, dK, dV)
    with pytest.raises(fa.FlexAttnError) as e:
        fa.flexattn_backward_stored(*args, n_blocks, torch.empty(need - 1, dtype=torch.uint8, device=DEV))
    assert e.value.status == fa.ERR_WORKSPACE
    with pytest.raises(fa.FlexAttnError) as e:
        fa.flexattn_backward_stored(*args, n_blocks, torch.empty(need + 64, dtype=torch.uint8, device=DEV)[16:])
    assert e.value.status == fa.ERR_INVALID_ARG
    small = 3
    ws = torch.zeros(fa.flexattn_backward_stored_workspace_bytes(Q, K, bm, small), dtype=torch.uint8, device=DEV)
    fa.flexattn_backward_stored(*args, small, ws)
    torch.cuda.synchronize()
    assert torch.isfinite(dQ.float()).all() and torch.isfinite(dK.float()).all() and torch.isfinite(dV.float()).all()


def test_stored_strided_layout_and_stages_agree():
    """[B, S, H, D] memory layout for every tensor, and the stages run one by one on one workspace, give bit
    for bit what the dense single call gives."""
    import paper_2412_05496_amd as fa
    wl = SMALL["cfg2_small"].scaled(S=1000, Hq=4, Hkv=2)          # a cut last block and GQA as well
    inp = wlm.make_train_inputs(wl, with_dO=True)
    O, LSE, bm, ids = run_forward(wl, inp, DEV)
    dQ, dK, dV = run_backward(wl, inp, DEV, O, LSE, bm, ids, stored=True)
    mask_id, score_id, params, Q, K, V = ids
    bshd = lambda t: t.transpose(1, 2).contiguous().transpose(1, 2)
    Qs, Ks, Vs, Os, dOs = (bshd(t) for t in (Q, K, V, O, inp.dO.to(DEV)))
    dQs, dKs, dVs = (bshd(torch.full_like(t, float("nan"))) for t in (Q, K, V))
    n_blocks = nonempty_blocks(bm)
    ws = torch.empty(fa.flexattn_backward_stored_workspace_bytes(Q, K, bm, n_blocks), dtype=torch.uint8, device=DEV)
    for stage in (fa.BWD_DELTA, fa.BWD_DKDV, fa.BWD_DQ):
        fa.flexattn_backward_stored(Qs, Ks, Vs, Os, dOs, LSE, score_id, mask_id, params, bm, inp.scale,
                                    dQs if stage == fa.BWD_DQ else None, dKs if stage == fa.BWD_DKDV else None,
                                    dVs if stage == fa.BWD_DKDV else None, n_blocks, ws, stage)
    torch.cuda.synchronize()
    assert torch.equal(dQs, dQ) and torch.equal(dKs, dK) and torch.equal(dVs, dV)
