"""MI355X-native fused LoRA linear layer (forward + backward, single and multi adapter).

The compute lives in the HIP library built from csrc/ (C ABI declared in include/lorafusion.h);
`binding` marshals arguments to it.  There is no CPU fallback: calling an op without the
built library raises.
"""
