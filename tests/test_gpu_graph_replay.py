"""The entry points under HIP graph capture: the library allocates nothing, waits for nothing and clears
memory with kernels only, so a whole step (BlockMask build, forward, both backwards) and a paged decode
can be recorded once and replayed.  Every replay is checked bit for bit against the eager result on
the same inputs, with eager work and synchronisations between replays and with the inputs rewritten in
place (the graph holds addresses, not values)."""
import pytest
import torch

import flex_workloads as wlm
from helpers import library_mods

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def nan_like(t):
    return torch.full_like(t, float("nan"))


class TrainStep:
    """Buffers of one training step at fixed addresses, and the step itself on the current stream."""

    def __init__(self, wl, inp):
        import paper_2412_05496_amd as fa
        self.fa, self.wl = fa, wl
        self.mask_id, self.score_id, self.params, Bm = library_mods(wl, inp, DEV)
        self.scale = inp.scale
        self.Q, self.K, self.V, self.dO = (t.to(DEV).clone() for t in (inp.Q, inp.K, inp.V, inp.dO))
        self.bm = fa.alloc_blockmask(Bm, 1, wl.S, wl.S, wl.Bq, wl.Bk, device=DEV)
        self.bm_ws = torch.empty(max(fa.flexattn_blockmask_workspace_bytes(Bm, 1, wl.S, wl.S, wl.Bq, wl.Bk), 1),
                                 dtype=torch.uint8, device=DEV)
        self.O, self.LSE = nan_like(self.Q), torch.empty(self.Q.shape[:3], dtype=torch.float32, device=DEV)
        self.grads = [nan_like(t) for t in (self.Q, self.K, self.V)]            # dS kept in memory
        self.grads_rc = [nan_like(t) for t in (self.Q, self.K, self.V)]         # dS recomputed
        # no host read of the block count is possible inside a capture: size for every block of the grid
        self.n_blocks = Bm * (-(-wl.S // wl.Bq)) * (-(-wl.S // wl.Bk))
        self.ws_st = torch.empty(fa.flexattn_backward_stored_workspace_bytes(self.Q, self.K, self.bm, self.n_blocks),
                                 dtype=torch.uint8, device=DEV)
        self.ws_rc = torch.empty(max(fa.flexattn_backward_workspace_bytes(self.Q, self.K), 1), dtype=torch.uint8,
                                 device=DEV)

    def outputs(self):
        return [self.O, self.LSE, *self.grads, *self.grads_rc]

    def poison(self):
        for t in self.outputs():
            t.fill_(float("nan"))

    def run(self):
        fa = self.fa
        fa.flexattn_blockmask_build(self.mask_id, self.params, self.bm, self.bm_ws)
        fa.flexattn_forward(self.Q, self.K, self.V, self.score_id, self.mask_id, self.params, self.bm, self.scale,
                            self.O, self.LSE)
        fa.flexattn_backward_stored(self.Q, self.K, self.V, self.O, self.dO, self.LSE, self.score_id, self.mask_id,
                                    self.params, self.bm, self.scale, *self.grads, self.n_blocks, self.ws_st)
        fa.flexattn_backward(self.Q, self.K, self.V, self.O, self.dO, self.LSE, self.score_id, self.mask_id,
                             self.params, self.bm, self.scale, *self.grads_rc, self.ws_rc)


def eager_work():
    a = torch.randn(512, 512, device=DEV)
    (a @ a).sum().item()


@pytest.mark.parametrize("mask,score,S,D", [("causal", "softcap", 1000, 128), ("doc_causal", "alibi", 1536, 64)])
def test_training_step_replays_bit_exactly(mask, score, S, D):
    wl = wlm.CFG2.scaled(B=2, Hq=4, Hkv=2, S=S, D=D, mask=mask, score=score, softcap=20.0, seed=31,
                         doc_len_min=100, doc_len_max=700)
    print(f"[case] graph replay of a training step: {mask}/{score} S={S} D={D}", flush=True)
    step = TrainStep(wl, wlm.make_train_inputs(wl, with_dO=True))
    fresh = [wlm.make_train_inputs(wl.scaled(seed=31 + i), with_dO=True) for i in (1, 2)]

    def load(inp):
        for dst, src in ((step.Q, inp.Q), (step.K, inp.K), (step.V, inp.V), (step.dO, inp.dO)):
            dst.copy_(src.to(DEV))
        if inp.doc_ids is not None:                # other documents: the BlockMask changes with them
            step.params.doc_ids.copy_(inp.doc_ids.to(DEV))

    step.run()                                     # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step.run()
    torch.cuda.synchronize()

    for round_, inp in enumerate([None, fresh[0], fresh[1], fresh[0]]):
        if inp is not None:
            load(inp)
        step.poison()
        step.run()
        torch.cuda.synchronize()
        want = [t.clone() for t in step.outputs()]
        assert all(torch.isfinite(t.float()).all() for t in want)
        eager_work()
        step.poison()
        graph.replay()
        torch.cuda.synchronize()
        for i, (got, ref) in enumerate(zip(step.outputs(), want)):
            assert torch.equal(got, ref), f"replay {round_}, output {i}"
        eager_work()


def test_paged_decode_replays_bit_exactly_with_lengths_changed_in_place():
    import paper_2412_05496_amd as fa
    wl = wlm.CFG5.scaled(B=6, ctx_min=100, ctx_max=5000, max_pages=320, seed=5)
    inp = wlm.make_decode_inputs(wl)
    print(f"[case] graph replay of paged decode: ctx {inp.ctx_lens.tolist()}", flush=True)
    Q, Kp, Vp = inp.Q.to(DEV), inp.K_pool.to(DEV), inp.V_pool.to(DEV)
    pt, ctx = inp.page_table.to(DEV), inp.ctx_lens.to(DEV).clone()
    params = fa.ModParams(softcap=30.0)
    ws = torch.empty(max(fa.flexattn_paged_decode_workspace_bytes(Q, Kp, pt), 1), dtype=torch.uint8, device=DEV)
    outs = {name: (torch.empty((Q.shape[0], Q.shape[1], Q.shape[-1]), dtype=torch.bfloat16, device=DEV),
                   torch.empty((Q.shape[0], Q.shape[1]), dtype=torch.float32, device=DEV))
            for name in ("ws", "static")}

    def run():
        fa.flexattn_paged_decode(Q, Kp, Vp, pt, ctx, fa.SCORE_SOFTCAP, fa.MASK_CTX_LEN, params, inp.scale,
                                 *outs["ws"], ws)
        fa.flexattn_paged_decode_static(Q, Kp, Vp, pt, ctx, fa.SCORE_SOFTCAP, fa.MASK_CTX_LEN, params, inp.scale,
                                        *outs["static"])

    def poison():
        for O, L in outs.values():
            O.fill_(float("nan"))
            L.fill_(float("nan"))

    run()                                          # also takes the static array's address, outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    torch.cuda.synchronize()

    lens0 = inp.ctx_lens.clone()
    for round_, lens in enumerate([lens0, (lens0 // 2).clamp(min=1), torch.ones_like(lens0), lens0]):
        ctx.copy_(lens.to(DEV))
        Q.copy_((inp.Q.float() * (1.0 + 0.25 * round_)).to(torch.bfloat16).to(DEV))
        poison()
        run()
        torch.cuda.synchronize()
        want = [t.clone() for pair in outs.values() for t in pair]
        assert all(torch.isfinite(t.float()).all() for t in want)
        eager_work()
        poison()
        graph.replay()
        torch.cuda.synchronize()
        got = [t for pair in outs.values() for t in pair]
        for i, (g, r) in enumerate(zip(got, want)):
            assert torch.equal(g, r), f"replay {round_}, output {i}"
