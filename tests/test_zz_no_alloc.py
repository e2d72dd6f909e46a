"""multi_lora_bwd_static: the backward for callers that cannot allocate (its workspace is a static device array of the
library).  Called through the C ABI twice in a row, the second time on a smaller input, and compared bit for bit with
multi_lora_bwd on a caller-allocated workspace (both run the same kernels in the same order, and every reduction has a
fixed order, so equal bits is the bar) and with the CPU oracle to the usual tolerance."""
import numpy as np
import pytest
import torch

from oracle import multilora_oracle as orc
from paper_2604_05426_amd import binding as ml
from paper_2604_05426_amd import workloads as wl
from paper_2604_05426_amd.harness import DeviceLayer, to_host
from util import rel_fro

pytestmark = pytest.mark.gpu


def run_both(w):
    print(f"[case] bwd_static {w.name} dtype={w.dtype} T={w.T} k={w.k} n={w.n} ranks={w.ranks} lens={w.seg_lens}", flush=True)
    dl = DeviceLayer(w)
    assert dl.plan.workspace_bytes() <= ml.STATIC_WORKSPACE_BYTES
    dl.forward()
    dl.backward()
    dl.sync()
    want = [t.clone() for t in (dl.dX, *dl.dA, *dl.dB)]
    for t in (dl.dX, *dl.dA, *dl.dB):
        t.fill_(float("nan"))
    dl.workspace.fill_(0xFF)          # the caller's workspace must play no part in the static call
    ws_before = dl.workspace.clone()
    ml.multi_lora_bwd_static(dl.plan, dl.dY, dl.X, dl.W, dl.A, dl.B, dl.S, dl.dX, dl.dA, dl.dB, 0, dl.stream)
    dl.sync()
    assert torch.equal(dl.workspace, ws_before)
    for got, ref in zip((dl.dX, *dl.dA, *dl.dB), want):
        assert torch.equal(got.view(torch.uint8), ref.view(torch.uint8))
    bw = orc.backward(w.dY, w.X, w.W, w.A, w.B, w.scales, w.offsets)
    tol = 1e-2 if w.dtype == "bf16" else 1e-5
    assert rel_fro(to_host(dl.dX), bw.dX) <= tol
    for i in range(w.N):
        assert rel_fro(to_host(dl.dA[i]), bw.dA[i]) <= tol and rel_fro(to_host(dl.dB[i]), bw.dB[i]) <= tol
    return dl


def test_static_workspace_backward_two_calls_second_smaller():
    # first call: a segment split over several weight-gradient chunks (fp32 partials in the workspace), a wide rank,
    # an empty adapter; second call: a smaller layer whose dS and partials land on top of the first call's leftovers
    big = wl.small_case(seed=91, dtype="bf16", k=1024, n=512, ranks=(8, 8, 16, 64, 100, 0), seg_lens=(256, 256, 512, 1300, 90, 7),
                        scales=(2.0, 0.5, 1.0, 0.25, 0.125, 1.0), b_sigma=0.3)
    small = wl.small_case(seed=92, dtype="bf16", k=256, n=320, ranks=(16, 4, 33), seg_lens=(700, 65, 129),
                          scales=(1.0, 2.0, 0.5), b_sigma=0.3)
    a = run_both(big)
    b = run_both(small)
    # and the fp32 path through the same entry point
    run_both(wl.config(0))
    a.plan.destroy(); b.plan.destroy()


def test_static_workspace_backward_rejects_oversized_plans_and_bad_arguments():
    # dS alone (300 000 tokens x rank 128 in bf16 = 76.8 MB) exceeds the static array; the call is rejected before any
    # pointer is looked at and nothing is launched
    T = 300_000
    plan = ml.Plan(ml.BF16, T, 64, 64, [128], [1.0], [0, T])
    print(f"[case] oversized plan: workspace {plan.workspace_bytes()} bytes", flush=True)
    assert plan.workspace_bytes() > ml.STATIC_WORKSPACE_BYTES
    with pytest.raises(ml.MultiLoraError) as e:
        ml.multi_lora_bwd_static(plan, 256, 256, 256, [256], [256], 256, 256, [256], [256])
    assert e.value.status == -7 and "static workspace" in str(e.value)
    plan.destroy()
    assert ml.lib().multi_lora_bwd_static(None, None, None, None, None, None, None, None, None, None, 0, None) == -1


def test_static_workspace_backward_inside_a_captured_graph():
    """The callers this entry point is for: a step captured into a HIP graph (no allocation, no workspace to carry).  The
    replays must reproduce the eager result bit for bit, with eager work of the same plan in between."""
    w = wl.small_case(seed=93, dtype="bf16", k=256, n=320, ranks=(8, 64, 100, 16), seg_lens=(300, 700, 77, 0),
                      scales=(2.0, 0.25, 1.0, 3.0), b_sigma=0.3)
    dl = DeviceLayer(w)
    outs = lambda: [dl.Y, dl.dX, dl.S] + [t for t in dl.dA + dl.dB if t.numel()]
    dl.forward(); dl.backward(); dl.sync()
    ref = [t.clone() for t in outs()]
    eager_stream = dl.stream
    graph, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
    with torch.cuda.graph(graph, stream=side):
        st = torch.cuda.current_stream().cuda_stream
        ml.multi_lora_fwd(dl.plan, dl.X, dl.W, dl.A, dl.B, dl.Y, dl.S, None, 0, st)
        ml.multi_lora_bwd_static(dl.plan, dl.dY, dl.X, dl.W, dl.A, dl.B, dl.S, dl.dX, dl.dA, dl.dB, 0, st)
    for rep in range(3):
        for t in outs():
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, want in zip(outs(), ref):
            assert torch.equal(got.view(torch.uint8), want.view(torch.uint8)), rep
        dl.forward(ml.FLAG_BASE_ONLY); dl.backward(); dl.sync()      # eager work between the replays, caller's workspace
    dl.plan.destroy()
