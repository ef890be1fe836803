"""CPU oracle for the LoRA-adapted linear layer (test infrastructure, not product code).

Only the tests, the smoke check and the benchmark's CPU-baseline leg may import this package.
It shares no code with the HIP library and never imports it.
"""
from .lora_oracle import (  # noqa: F401
    dropout_threshold,
    dropout_scale,
    dropout_words,
    keep_mask,
    lora_fwd,
    lora_bwd,
    multi_lora_fwd,
    multi_lora_bwd,
)
