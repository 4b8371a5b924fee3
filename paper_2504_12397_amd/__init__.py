"""libalora: Activated-LoRA prefill/decode over a reused base-model KV cache, hand-written
HIP for gfx950 behind a C ABI (include/alora.h).  The Python side only marshals arguments."""
