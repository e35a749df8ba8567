"""GPU parity for sequence lengths that are no multiple of the block size: the last row / column of
BlockMask blocks is cut by the edge of the score matrix (BlockMask bit for bit, forward, backward)."""
import pytest
import torch

import flex_workloads as wlm
from oracle import flex_oracle as fo
from tests import helpers as hp

pytestmark = pytest.mark.gpu

CASES = [
    # name, base workload, overrides, q_len (None = S)
    ("causal_softcap_d128_s1000", wlm.CFG2, dict(B=1, Hq=2, Hkv=2, S=1000), None),
    ("none_d64_300x777_bk128", wlm.CFG1, dict(B=1, Hq=2, Hkv=1, S=777, D=64, Bq=64, Bk=128, mask="none", backward=True), 300),
    ("causal_d64_q1_kv65", wlm.CFG1, dict(B=2, Hq=2, Hkv=2, S=65, backward=True), 1),
    ("doc_alibi_d64_s1000", wlm.CFG3, dict(B=2, Hq=4, Hkv=4, S=1000, doc_len_min=50, doc_len_max=400), None),
    ("swa_prefix_relbias_gqa_d128_s999", wlm.CFG4, dict(B=1, Hq=4, Hkv=2, S=999, window=200, prefix_len=100, rel_len=64), None),
    ("causal_d128_s130_bq128", wlm.CFG2, dict(B=1, Hq=1, Hkv=1, S=130, score="identity"), None),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_ragged_lengths(case):
    import paper_2412_05496_amd as fa
    name, base, over, q_len = case
    dev = torch.device("cuda:0")
    wl = base.scaled(name="ragged_" + name, seed=3500 + len(name), **over)
    inp = wlm.make_train_inputs(wl, with_dO=True)
    Lq = wl.S if q_len is None else q_len
    Q, dO = inp.Q[:, :, :Lq].contiguous(), inp.dO[:, :, :Lq].contiguous()
    score_mod, mask_mod = hp.oracle_mods(wl, inp)
    O_ref, LSE_ref = fo.flex_attention(Q, inp.K, inp.V, score_mod, mask_mod, inp.scale)
    dQ_ref, dK_ref, dV_ref = fo.flex_attention_backward(Q, inp.K, inp.V, dO, score_mod, mask_mod, inp.scale)

    mask_id, score_id, params, Bm = hp.library_mods(wl, inp, dev)
    bm = fa.alloc_blockmask(Bm, 1, Lq, wl.S, wl.Bq, wl.Bk, device=dev)
    fa.flexattn_blockmask_build(mask_id, params, bm)
    torch.cuda.synchronize()
    hp.assert_blockmask_equal(bm, fo.create_block_mask(mask_mod, Bm, 1, Lq, wl.S, wl.Bq, wl.Bk))

    # guard rows / keys right behind the tensors: the kernels must not write past the real lengths
    def padded(t, rows):
        buf = torch.full((t.shape[0], t.shape[1], rows + 64, t.shape[3]), 7.0, dtype=t.dtype, device=dev)
        return buf, buf[:, :, :rows]
    Qd, Kd, Vd, dOd = Q.to(dev), inp.K.to(dev), inp.V.to(dev), dO.to(dev)
    O_buf, O = padded(Qd, Lq)
    dQ_buf, dQ = padded(Qd, Lq)
    dK_buf, dK = padded(Kd, wl.S)
    dV_buf, dV = padded(Vd, wl.S)
    LSE = torch.full(Qd.shape[:3], float("nan"), dtype=torch.float32, device=dev)
    fa.flexattn_forward(Qd, Kd, Vd, score_id, mask_id, params, bm, inp.scale, O, LSE)
    fa.flexattn_backward(Qd, Kd, Vd, O, dOd, LSE, score_id, mask_id, params, bm, inp.scale, dQ, dK, dV)
    torch.cuda.synchronize()
    hp.check_output(O, LSE, O_ref, LSE_ref)
    hp.check_grad("dQ", dQ, dQ_ref)
    hp.check_grad("dK", dK, dK_ref)
    hp.check_grad("dV", dV, dV_ref)
    for buf, rows in ((O_buf, Lq), (dQ_buf, Lq), (dK_buf, wl.S), (dV_buf, wl.S)):
        assert (buf[:, :, rows:] == 7.0).all()
