"""MI355X-native routed-LoRA hot path (MoLoRA, per-token adapter routing).

The compute lives in the HIP library under csrc/, reached through the C ABI declared
in include/molora.h; `binding` marshals torch tensors into it.  Importing the package
does not load the library; the first call does, and fails loudly if it is not built.
"""
__all__ = ["binding", "workloads"]
