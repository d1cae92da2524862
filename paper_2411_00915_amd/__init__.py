"""MI355X-native heterogeneous-LoRA batching operator (hot path of VaLoRA's ATMM,
paper section 4.3):  y = x W + s_a (x A_a) B_a  for tokens tagged with adapters.

`paper_2411_00915_amd.binding` is the thin ctypes layer over the C-ABI library
(include/lora_abi.h); `paper_2411_00915_amd.workloads` draws seeded inputs.
"""
__all__ = ["binding", "workloads", "build"]
