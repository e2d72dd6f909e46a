"""Device-side plumbing around the C ABI: upload a Workload, allocate outputs with torch,
call multi_lora_fwd / multi_lora_bwd, fetch results.  No arithmetic of the layer happens here.
"""
from __future__ import annotations

from typing import List, Optional

import numpy as np
import torch

from . import binding as ml
from .workloads import Workload, bf16_bits


def to_device(a: np.ndarray, dtype: str, device, nan_guard: bool = False) -> torch.Tensor:
    """float32 host array (holding values exact in `dtype`) -> device tensor of that dtype.  With `nan_guard` the tensor
    is a view into a larger allocation whose head and tail are NaN: a kernel that reads past either end of an input and
    lets the value reach an output poisons that output, which the parity checks then catch."""
    if dtype == "bf16":
        bits = bf16_bits(a).view(np.int16)
        t = torch.from_numpy(bits).to(device).view(torch.bfloat16)
    else:
        t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)
    if not nan_guard:
        return t
    buf = torch.full((t.numel() + 2 * GUARD_ELEMS,), float("nan"), dtype=t.dtype, device=device)
    view = buf[GUARD_ELEMS:GUARD_ELEMS + t.numel()].view(t.shape)
    view.copy_(t)
    return view


def to_host(t: torch.Tensor) -> np.ndarray:
    """device tensor -> float64 numpy (exact widening)."""
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


GUARD_ELEMS = 4096          # guard region either side of every output (elements of the output's dtype)
GUARD_VALUE = -7.0          # exact in bf16 and fp32; 0xA5 for the byte-typed workspace


class DeviceLayer:
    """One multi-LoRA layer resident on the GPU: inputs, outputs, plan and workspace.

    With ``guards`` (the default) every output the library writes -- Y, dX, S, dA_i, dB_i and the workspace -- sits
    inside a larger allocation between two guard regions filled with a known value; ``check_guards`` (called by
    ``sync``) asserts that no kernel wrote outside the tensor it was given.  The inputs (X, W, dY, A_i, B_i) sit between
    NaN regions, so that a value read from outside an input cannot reach an output unnoticed."""

    def __init__(self, w: Workload, device: str = "cuda:0", canary: Optional[float] = None,
                 like: Optional["ml.Plan"] = None, guards: bool = True):
        if not torch.cuda.is_available():
            raise RuntimeError("DeviceLayer needs a GPU; there is no CPU fallback")
        self.w = w
        self.device = torch.device(device)
        self.tdtype = torch.bfloat16 if w.dtype == "bf16" else torch.float32
        self.mdtype = ml.BF16 if w.dtype == "bf16" else ml.F32
        dev, dt = self.device, w.dtype
        ng = guards        # inputs sit between NaN regions, outputs between regions of a known value
        self.X, self.W, self.dY = to_device(w.X, dt, dev, ng), to_device(w.W, dt, dev, ng), to_device(w.dY, dt, dev, ng)
        self.A = [to_device(a, dt, dev, ng) for a in w.A]
        self.B = [to_device(b, dt, dev, ng) for b in w.B]
        fill = float("nan") if canary is None else canary
        self._guarded = []

        def out(name, *shape):
            if not guards:
                return torch.full(shape, fill, dtype=self.tdtype, device=dev)
            numel = int(np.prod(shape))
            buf = torch.full((numel + 2 * GUARD_ELEMS,), GUARD_VALUE, dtype=self.tdtype, device=dev)
            view = buf[GUARD_ELEMS:GUARD_ELEMS + numel].view(*shape)
            view.fill_(fill)
            self._guarded.append((name, buf, numel, GUARD_VALUE))
            return view

        self.Y, self.dX = out("Y", w.T, w.n), out("dX", w.T, w.k)
        self.S = out("S", max(w.R1, 1))
        self.dA = [out(f"dA{i}", w.k, r) for i, r in enumerate(w.ranks)]
        self.dB = [out(f"dB{i}", r, w.n) for i, r in enumerate(w.ranks)]
        self.stream = torch.cuda.current_stream(dev).cuda_stream
        if like is None:
            self.plan = ml.Plan(self.mdtype, w.T, w.k, w.n, w.ranks, w.scales, w.offsets, stream=self.stream)
        else:      # another layer shape over the segmentation tables of an existing plan
            self.plan = ml.Plan.like(like, w.k, w.n, stream=self.stream)
        self.ws_bytes = self.plan.workspace_bytes()
        ws_len = max(self.ws_bytes, 256)
        if guards:
            buf = torch.full((ws_len + 2 * GUARD_ELEMS,), 0xA5, dtype=torch.uint8, device=dev)
            self.workspace = buf[GUARD_ELEMS:GUARD_ELEMS + ws_len]
            self.workspace.zero_()
            self._guarded.append(("workspace", buf, ws_len, 0xA5))
        else:
            self.workspace = torch.zeros(ws_len, dtype=torch.uint8, device=dev)

    def check_guards(self) -> None:
        """No kernel may have written outside the outputs it was handed."""
        for name, buf, numel, value in self._guarded:
            head, tail = buf[:GUARD_ELEMS], buf[GUARD_ELEMS + numel:]
            if not (bool(torch.all(head == value)) and bool(torch.all(tail == value))):
                raise AssertionError(f"guard region around {name} was overwritten")

    @classmethod
    def synthetic(cls, name: str, dtype: str, k: int, n: int, ranks, seg_lens, scales, seed: int,
                  device: str = "cuda:0", like: Optional["ml.Plan"] = None) -> "DeviceLayer":
        """Same shapes and value distributions as workloads.make_workload, drawn on the GPU (no host copy, hence
        nothing an oracle could be run on): for timing layers too large to generate on the host in reasonable time."""
        if not torch.cuda.is_available():
            raise RuntimeError("DeviceLayer needs a GPU; there is no CPU fallback")
        self = cls.__new__(cls)
        self._guarded = []
        off = [0]
        for t in seg_lens:
            off.append(off[-1] + int(t))
        T = off[-1]
        self.w = Workload(name=name, dtype=dtype, T=T, k=k, n=n, ranks=[int(r) for r in ranks],
                          scales=[float(x) for x in scales], offsets=off, X=None, W=None, A=[], B=[], dY=None, seed=seed)
        self.device = torch.device(device)
        self.tdtype = torch.bfloat16 if dtype == "bf16" else torch.float32
        self.mdtype = ml.BF16 if dtype == "bf16" else ml.F32
        gen = torch.Generator(device=self.device).manual_seed(seed)

        def draw(shape, sigma):
            return (torch.randn(shape, generator=gen, device=self.device, dtype=torch.float32) * sigma).to(self.tdtype)

        self.X, self.W, self.dY = draw((T, k), 1.0), draw((k, n), 0.02), draw((T, n), 1.0)
        self.A = [draw((k, r), 1.0 / np.sqrt(k)) for r in self.w.ranks]
        self.B = [draw((r, n), 0.02) for r in self.w.ranks]
        self.Y = torch.zeros((T, n), dtype=self.tdtype, device=self.device)
        self.dX = torch.zeros((T, k), dtype=self.tdtype, device=self.device)
        self.S = torch.zeros(max(self.w.R1, 1), dtype=self.tdtype, device=self.device)
        self.dA = [torch.zeros((k, r), dtype=self.tdtype, device=self.device) for r in self.w.ranks]
        self.dB = [torch.zeros((r, n), dtype=self.tdtype, device=self.device) for r in self.w.ranks]
        self.stream = torch.cuda.current_stream(self.device).cuda_stream
        if like is None:
            self.plan = ml.Plan(self.mdtype, T, k, n, self.w.ranks, self.w.scales, off, stream=self.stream)
        else:
            self.plan = ml.Plan.like(like, k, n, stream=self.stream)
        self.ws_bytes = self.plan.workspace_bytes()
        self.workspace = torch.zeros(max(self.ws_bytes, 256), dtype=torch.uint8, device=self.device)
        return self

    def forward(self, flags: int = 0) -> None:
        ml.multi_lora_fwd(self.plan, self.X, self.W, self.A, self.B, self.Y, self.S, self.workspace,
                          flags, self.stream)

    def backward(self, flags: int = 0) -> None:
        ml.multi_lora_bwd(self.plan, self.dY, self.X, self.W, self.A, self.B, self.S, self.dX,
                          self.dA, self.dB, self.workspace, flags, self.stream)

    def sync(self) -> None:
        torch.cuda.synchronize(self.device)
        self.check_guards()

    # ---- results as float64 numpy ------------------------------------------------------
    def S_list(self) -> List[np.ndarray]:
        s = to_host(self.S)
        out, o = [], 0
        for t, r in zip(self.w.seg_lens, self.w.ranks):
            out.append(s[o:o + t * r].reshape(t, r))
            o += t * r
        return out

    def dS_list(self) -> List[np.ndarray]:
        esz = 2 if self.w.dtype == "bf16" else 4
        raw = self.workspace[: self.w.R1 * esz].view(self.tdtype) if self.w.R1 else self.workspace[:0].view(self.tdtype)
        s = to_host(raw)
        out, o = [], 0
        for t, r in zip(self.w.seg_lens, self.w.ranks):
            out.append(s[o:o + t * r].reshape(t, r))
            o += t * r
        return out


class DeviceBlock:
    """The LoRA'd linear layers of one transformer block over one segmentation: the first layer's plan is built from
    the metadata, every other layer's plan with multi_lora_plan_create_like on it.  `step` runs every forward, every
    backward (reverse order) and, when optimizer state was set up, the grouped AdamW update of every layer."""

    def __init__(self, layers: List[Workload], device: str = "cuda:0", canary: Optional[float] = None,
                 share_tables: bool = True):
        self.layers: List[DeviceLayer] = []
        for w in layers:
            base = self.layers[0].plan if (self.layers and share_tables) else None
            self.layers.append(DeviceLayer(w, device, canary, like=base))
        self.state = None

    @classmethod
    def synthetic(cls, dtype: str, shapes, ranks, seg_lens, scales, seed: int, device: str = "cuda:0") -> "DeviceBlock":
        """Layers drawn on the GPU (timing only), plans shared as in __init__."""
        self = cls.__new__(cls)
        self.layers, self.state = [], None
        for l, (name, k, n) in enumerate(shapes):
            base = self.layers[0].plan if self.layers else None
            self.layers.append(DeviceLayer.synthetic(name, dtype, k, n, ranks, seg_lens, scales, seed + l, device, like=base))
        return self

    def init_adamw(self) -> None:
        dev = self.layers[0].device
        self.state = []
        for dl in self.layers:
            sA = [torch.empty(3 * a.numel(), dtype=torch.float32, device=dev) for a in dl.A]
            sB = [torch.empty(3 * b.numel(), dtype=torch.float32, device=dev) for b in dl.B]
            ml.multi_lora_adamw_init(dl.plan, dl.A, dl.B, sA, sB, dl.stream)
            self.state.append((sA, sB))

    def step(self, hparams=None) -> None:
        for dl in self.layers:
            dl.forward()
        for dl in reversed(self.layers):
            dl.backward()
        if self.state is not None and hparams is not None:
            for dl, (sA, sB) in zip(self.layers, self.state):
                ml.multi_lora_adamw_step(dl.plan, dl.A, dl.B, dl.dA, dl.dB, sA, sB, hparams, dl.stream)

    def sync(self) -> None:
        self.layers[0].sync()
