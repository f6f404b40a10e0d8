"""MI355X-native fused multi-LoRA linear layer (tLoRA hot path).

`paper_2602_07263_amd.tlora` is the thin ctypes binding of the C-ABI library `libtlora.so`
(hand-written gfx950 kernels); `paper_2602_07263_amd.workloads` draws the seeded synthetic inputs.
Nothing here computes on the CPU: without the built library and a gfx950 device the binding raises.
"""
__all__ = ["tlora", "workloads", "build"]
