"""MI355X-native tree-verification pass of Spec-VLA (relaxed-acceptance speculative decoding).

`paper_2507_22424_amd.binding` is the thin ctypes layer over the C-ABI library
libspecvla_verify (hand-written HIP for gfx950); `paper_2507_22424_amd.workload`
draws the seeded synthetic inputs.  Nothing here falls back to the CPU.
"""

__all__ = ["binding", "workload"]
