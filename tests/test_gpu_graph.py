"""multi_lora_fwd / multi_lora_bwd only launch kernels, so a caller may capture them into a HIP graph (launch-bound
small layers).  The captured step is replayed several times, with eager work of the same plan and synchronisations in
between, and every replay must reproduce the eager result bit for bit."""
import pytest
import torch

from paper_2604_05426_amd import binding as ml
from paper_2604_05426_amd import workloads as wl
from paper_2604_05426_amd.harness import DeviceLayer

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_captured_step_replays_bit_identically(dtype):
    w = wl.small_case(seed=90, dtype=dtype, k=256, n=320, ranks=(8, 64, 100, 16), seg_lens=(300, 700, 77, 0),
                      scales=(2.0, 0.25, 1.0, 3.0), b_sigma=0.3)
    dl = DeviceLayer(w)
    outs = lambda: [dl.Y, dl.dX, dl.S] + [t for t in dl.dA + dl.dB if t.numel()]
    dl.forward(); dl.backward(); dl.sync()
    ref = [t.clone() for t in outs()]
    eager_stream = dl.stream

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.graph(graph, stream=side):
        dl.stream = torch.cuda.current_stream().cuda_stream      # the capturing stream
        dl.forward(); dl.backward()
    dl.stream = eager_stream
    for rep in range(4):
        for t in outs():
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, want in zip(outs(), ref):
            assert torch.equal(got.view(torch.uint8), want.view(torch.uint8)), rep
        # the program's own eager work between replays: the same plan on the ordinary stream, other flags
        dl.forward(ml.FLAG_BASE_ONLY); dl.backward(ml.FLAG_ACCUM_GRADS); dl.sync()


def test_eager_calls_with_other_buffers_after_a_captured_step():
    """A replay of a captured step rewrites the plan's device pointer table with the captured buffers.  An eager call
    with OTHER buffers, made after such a replay, must still reach its own buffers (the call may not trust a host-side
    record of what it uploaded last)."""
    mk = lambda seed: wl.small_case(seed=seed, dtype="bf16", k=256, n=320, ranks=(8, 64, 100, 16), seg_lens=(300, 700, 77, 0),
                                    scales=(2.0, 0.25, 1.0, 3.0), b_sigma=0.3)
    d1, d2 = DeviceLayer(mk(93)), DeviceLayer(mk(94))
    outs = lambda d: [d.Y, d.dX, d.S] + [t for t in d.dA + d.dB if t.numel()]
    for d in (d1, d2):
        d.forward(); d.backward(); d.sync()
    ref1, ref2 = [t.clone() for t in outs(d1)], [t.clone() for t in outs(d2)]
    plan, eager_stream = d1.plan, d1.stream

    def eager_on_d2():        # d1's plan, d2's buffers (same segmentation, so the plan fits)
        ml.multi_lora_fwd(plan, d2.X, d2.W, d2.A, d2.B, d2.Y, d2.S, d1.workspace, 0, eager_stream)
        ml.multi_lora_bwd(plan, d2.dY, d2.X, d2.W, d2.A, d2.B, d2.S, d2.dX, d2.dA, d2.dB, d1.workspace, 0, eager_stream)

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.graph(graph, stream=side):
        d1.stream = torch.cuda.current_stream().cuda_stream
        d1.forward(); d1.backward()
    d1.stream = eager_stream
    for rep in range(3):
        for t in outs(d1) + outs(d2):
            t.fill_(float("nan"))
        eager_on_d2()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, want in zip(outs(d1), ref1):
            assert torch.equal(got.view(torch.uint8), want.view(torch.uint8)), rep
        for got, want in zip(outs(d2), ref2):
            assert torch.equal(got.view(torch.uint8), want.view(torch.uint8)), rep
        for t in outs(d1) + outs(d2):
            t.fill_(float("nan"))
        eager_on_d2()             # same pointers as the last eager call, but the replay has changed the table since
        torch.cuda.synchronize()
        for got, want in zip(outs(d2), ref2):
            assert torch.equal(got.view(torch.uint8), want.view(torch.uint8)), rep
        for t in (d1.Y, d1.dX):   # and nothing of d1 was written
            assert bool(torch.isnan(t).all())
    d1.check_guards(); d2.check_guards()
