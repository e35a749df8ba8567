"""The measurement aids run, finish and report rates of the right order of magnitude (they are what
bench.py quotes the kernels against), and their clock readout is a plausible core clock."""
import pytest
import torch

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _ms(fn, n=3):
    fn()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(n):
        fn()
    b.record()
    b.synchronize()
    return a.elapsed_time(b) / n


@pytest.mark.parametrize("valu_mix,random_operands", [(0, False), (0, True), (1, True), (2, True)])
def test_mfma_probe(valu_mix, random_operands):
    import paper_2412_05496_amd as fa
    sink = torch.zeros(4, dtype=torch.float32, device=DEV)
    clocks = torch.zeros(fa.flexattn_probe_mfma_waves(), 2, dtype=torch.int64, device=DEV)
    iters = 4000
    ms = _ms(lambda: fa.flexattn_probe_mfma(iters, sink, valu_mix, random_operands, clocks))
    tflops = fa.flexattn_probe_mfma_flops(iters) / (ms * 1e-3) / 1e12
    ck = clocks.cpu().double()
    ghz = float(ck[:, 0].sum() / (ck[:, 1].sum() * 10.0))
    print(f"  [probe] mix {valu_mix} random {random_operands}: {tflops:.0f} TFLOP/s at {ghz:.2f} GHz", flush=True)
    assert (ck > 0).all()
    assert 300.0 < tflops < 2600.0            # below the datasheet peak, far above anything a stalled launch gives
    assert 0.8 < ghz < 2.6                    # the chip's clock range
    assert float(sink.abs().sum()) == 0.0     # the sink is never really written


def test_stream_read_probe_and_bad_arguments():
    import paper_2412_05496_amd as fa
    sink = torch.zeros(4, dtype=torch.float32, device=DEV)
    src = torch.ones(1 << 30, dtype=torch.uint8, device=DEV)
    ms = _ms(lambda: fa.flexattn_probe_stream_read(src, sink))
    gbs = src.numel() / (ms * 1e-3) / 1e9
    print(f"  [probe] stream read {gbs:.0f} GB/s", flush=True)
    assert 1000.0 < gbs < 8000.0
    with pytest.raises(fa.FlexAttnError):
        fa.flexattn_probe_mfma(0, sink)
    with pytest.raises(fa.FlexAttnError):
        fa.flexattn_probe_mfma(10, sink, valu_mix=3)
