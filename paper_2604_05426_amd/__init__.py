"""MI355X-native fused multi-LoRA linear layer (forward + backward).

The compute lives in ``csrc/`` (hand-written HIP for gfx950 behind the C ABI declared in
``include/multi_lora.h``); ``binding`` is the ctypes front end with the same entry points,
``workloads`` the seeded synthetic inputs.  Importing the package loads nothing native;
``binding`` loads the shared library on first use and raises if it is missing.
"""
__all__ = ["binding", "workloads", "build"]
