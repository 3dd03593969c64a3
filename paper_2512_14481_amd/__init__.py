"""MI355X-native hot path of SASQ (static activation scaling for quantization-aware training).

`paper_2512_14481_amd.binding` is the thin Python face of the C-ABI library declared in
include/sasq.h (same entry-point names, argument marshalling only); `workloads` draws the
seeded synthetic LLaMA-2-shaped inputs.  There is no CPU fallback: calling the binding without
the built HIP library raises.
"""
__all__ = ["binding", "workloads"]
