"""Randomised parity sweep: seeded draws of (variant, head dimension, block sizes, lengths, GQA group),
each checked against the oracle — BlockMask bit for bit, forward, backward — through the C ABI.  The
lengths are drawn without regard to the block sizes, so most cases have a cut last block."""
import random

import pytest
import torch

import flex_workloads as wlm
from oracle import flex_oracle as fo
from tests import helpers as hp

pytestmark = pytest.mark.gpu

VARIANTS = [("none", "identity"), ("causal", "identity"), ("causal", "alibi"), ("causal", "softcap"),
            ("swa_causal", "identity"), ("prefix_lm", "identity"), ("doc_causal", "identity"),
            ("doc_causal", "alibi"), ("swa_causal_or_prefix", "rel_bias")]


def draw(seed):
    rng = random.Random(seed)
    mask, score = rng.choice(VARIANTS)
    G = rng.choice([1, 1, 2, 4])
    Hkv = rng.choice([1, 2])
    S = rng.randint(1, 700)
    Lq = S if mask != "none" and rng.random() < 0.7 else rng.randint(1, S)
    kw = dict(name=f"rand{seed}", B=rng.choice([1, 2]), Hq=Hkv * G, Hkv=Hkv, S=S, D=rng.choice([64, 128]),
              Bq=rng.choice([64, 128]), Bk=rng.choice([64, 128]), mask=mask, score=score, seed=4000 + seed,
              backward=True, softcap=rng.choice([5.0, 30.0, 60.0]), window=rng.randint(0, 300),
              prefix_len=rng.randint(0, 200), rel_len=rng.choice([1, 17, 64]),
              doc_len_min=rng.randint(1, 40), doc_len_max=rng.randint(40, 400))
    scale = rng.choice([None, None, 0.3, 0.02])       # None: 1 / sqrt(D)
    return wlm.CFG1.scaled(**kw), Lq, scale


@pytest.mark.parametrize("seed", range(40))
def test_random_shape(seed):
    import paper_2412_05496_amd as fa
    wl, Lq, scale = draw(seed)
    dev = torch.device("cuda:0")
    print(f"case {seed}: {wl.mask}/{wl.score} B={wl.B} Hq={wl.Hq} Hkv={wl.Hkv} Lq={Lq} S={wl.S} D={wl.D} "
          f"block={wl.Bq}x{wl.Bk} scale={scale}", flush=True)
    inp = wlm.make_train_inputs(wl, with_dO=True)
    if scale is not None:
        inp.scale = scale
    Q, dO = inp.Q[:, :, :Lq].contiguous(), inp.dO[:, :, :Lq].contiguous()
    score_mod, mask_mod = hp.oracle_mods(wl, inp)
    O_ref, LSE_ref = fo.flex_attention(Q, inp.K, inp.V, score_mod, mask_mod, inp.scale)
    dQ_ref, dK_ref, dV_ref = fo.flex_attention_backward(Q, inp.K, inp.V, dO, score_mod, mask_mod, inp.scale)

    mask_id, score_id, params, Bm = hp.library_mods(wl, inp, dev)
    bm = fa.alloc_blockmask(Bm, 1, Lq, wl.S, wl.Bq, wl.Bk, device=dev)
    fa.flexattn_blockmask_build(mask_id, params, bm)
    torch.cuda.synchronize()
    hp.assert_blockmask_equal(bm, fo.create_block_mask(mask_mod, Bm, 1, Lq, wl.S, wl.Bq, wl.Bk))
    Qd, Kd, Vd, dOd = Q.to(dev), inp.K.to(dev), inp.V.to(dev), dO.to(dev)
    O = torch.full_like(Qd, float("nan"))
    LSE = torch.full(Qd.shape[:3], float("nan"), dtype=torch.float32, device=dev)
    fa.flexattn_forward(Qd, Kd, Vd, score_id, mask_id, params, bm, inp.scale, O, LSE)
    dQ, dK, dV = torch.full_like(Qd, float("nan")), torch.full_like(Kd, float("nan")), torch.full_like(Vd, float("nan"))
    fa.flexattn_backward(Qd, Kd, Vd, O, dOd, LSE, score_id, mask_id, params, bm, inp.scale, dQ, dK, dV)
    torch.cuda.synchronize()
    hp.check_output(O, LSE, O_ref, LSE_ref)
    hp.check_grad("dQ", dQ, dQ_ref)
    hp.check_grad("dK", dK, dK_ref)
    hp.check_grad("dV", dV, dV_ref)
    # the same gradients with dS kept in memory: dK / dV from the same kernel, dQ from the stored blocks
    dQ2, dK2, dV2 = torch.full_like(Qd, float("nan")), torch.full_like(Kd, float("nan")), torch.full_like(Vd, float("nan"))
    fa.flexattn_backward_stored(Qd, Kd, Vd, O, dOd, LSE, score_id, mask_id, params, bm, inp.scale, dQ2, dK2, dV2,
                                hp.nonempty_blocks(bm))
    torch.cuda.synchronize()
    assert torch.equal(dK2, dK) and torch.equal(dV2, dV)
    hp.check_grad("dQ (dS kept in memory)", dQ2, dQ_ref)
