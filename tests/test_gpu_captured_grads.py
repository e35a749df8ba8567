"""GPU parity of the gradients of captured tensors (ALiBi bias per head, relative-bias table) against
the oracle, through the C ABI."""
import pytest
import torch

import flex_workloads as wlm
from oracle import flex_oracle as fo
from tests import helpers as hp

pytestmark = pytest.mark.gpu

CASES = [
    ("causal_alibi_d64_gqa", wlm.CFG3, dict(B=2, Hq=4, Hkv=2, S=512, mask="causal")),
    ("doc_alibi_d64", wlm.CFG3, dict(B=2, Hq=4, Hkv=4, S=1024, doc_len_min=60, doc_len_max=500)),
    ("swa_prefix_relbias_gqa_d128", wlm.CFG4, dict(B=2, Hq=4, Hkv=2, S=1024, window=300, prefix_len=100, rel_len=64)),
    ("relbias_d128_bq64_ragged", wlm.CFG4, dict(B=1, Hq=2, Hkv=2, S=1000, Bq=64, window=150, prefix_len=70, rel_len=256)),
    ("causal_alibi_d64_ragged", wlm.CFG3, dict(B=1, Hq=2, Hkv=1, S=333, mask="causal", Bq=64, Bk=128)),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_captured_gradients_match_oracle(case):
    import paper_2412_05496_amd as fa
    name, base, over = case
    dev = torch.device("cuda:0")
    wl = base.scaled(name="captured_" + name, seed=3600 + len(name), **over)
    inp = wlm.make_train_inputs(wl, with_dO=True)
    score_mod, mask_mod = hp.oracle_mods(wl, inp)
    ref = fo.flex_attention_backward_captured(inp.Q, inp.K, inp.V, inp.dO, score_mod, mask_mod, inp.scale)

    O, LSE, bm, (mask_id, score_id, params, Q, K, V) = hp.run_forward(wl, inp, dev)
    dO = inp.dO.to(dev)
    d_alibi = torch.full((wl.Hq,), float("nan"), device=dev) if "alibi_bias" in ref else None
    d_rel = torch.full((wl.Hq, wl.rel_len), float("nan"), device=dev) if "rel_bias" in ref else None
    for _ in range(2):      # written, not accumulated: a second call gives the same
        fa.flexattn_backward_captured(Q, K, V, O, dO, LSE, score_id, mask_id, params, bm, inp.scale, d_alibi, d_rel)
    torch.cuda.synchronize()
    # These sums run over EVERY (q, kv) pair of a head (the ALiBi one weighted by q - kv), so the
    # rounding of delta = rowsum(dO * O) from the bf16 O, which shifts all dS of a row the same way,
    # does not average out as it does in dQ / dK / dV: mean error <= 1e-2 of the mean magnitude.
    if d_alibi is not None:
        hp.check_grad("d_alibi_bias", d_alibi, ref["alibi_bias"], mean_tol=1e-2)
    if d_rel is not None:
        hp.check_grad("d_rel_bias", d_rel, ref["rel_bias"], mean_tol=1e-2)
        assert float(ref["rel_bias"].abs().max()) > 0


def test_score_mods_without_captured_tensors_are_refused():
    import paper_2412_05496_amd as fa
    dev = torch.device("cuda:0")
    wl = wlm.CFG1
    inp = wlm.make_train_inputs(wl, with_dO=True)
    O, LSE, bm, (mask_id, score_id, params, Q, K, V) = hp.run_forward(wl, inp, dev)
    with pytest.raises(fa.FlexAttnError):
        fa.flexattn_backward_captured(Q, K, V, O, inp.dO.to(dev), LSE, score_id, mask_id, params, bm, inp.scale)
