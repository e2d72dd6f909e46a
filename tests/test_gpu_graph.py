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
