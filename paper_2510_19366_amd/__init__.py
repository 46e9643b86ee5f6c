"""MI355X-native routed-expert forward of a sub-expert MoE layer with per-token k.

The compute lives in ``csrc/`` behind a C ABI (``include/moe_prism.h``);
``binding`` marshals torch device tensors into it.  Nothing is imported
eagerly so that ``workloads`` (input synthesis only) can be used without the
HIP library.
"""
__all__ = ["workloads", "binding"]
