"""MI355X-native dedup dispatch / combine for hierarchical MoE all-to-all (HierMoE, Eq.(7)).

The compute lives in ``libhiermoe.so`` (hand-written HIP for gfx950 behind a C ABI, declared in
``include/hiermoe.h``); ``binding`` marshals torch device tensors into it.  ``workloads`` only
generates seeded synthetic inputs.  Nothing here falls back to the CPU: without the built
library every call raises.
"""
__all__ = ["binding", "workloads"]
