"""MI355X-native routed-LoRA linear layers of MiLoRA (prompt-aware layer-level LoRA routing).

`binding` holds the Python face of the C-ABI library (`milora_route`,
`milora_routed_linear`, `milora_layer_decode`); `synth` draws the seeded
synthetic workloads.  Importing the package loads nothing native; the binding
loads the HIP library on first use and raises if it is missing.
"""
__all__ = ["binding", "synth"]
