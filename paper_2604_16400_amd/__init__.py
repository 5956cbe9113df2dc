"""MI355X-native mixed-batch LoRA linear layer (the hot path under CoLLM's co-execution of
LoRA inference and LoRA fine-tuning on one shared-weight replica).

``paper_2604_16400_amd.binding`` is the Python face of the C-ABI library built from
``csrc/``; ``paper_2604_16400_amd.workloads`` draws the seeded synthetic inputs.  Nothing is
imported eagerly so that the input generators can be used without the GPU library.
"""
__all__ = ["binding", "workloads"]
