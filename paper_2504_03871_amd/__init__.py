"""MoE expert layer (gate, dispatch, grouped expert FFN, combine; forward and backward) for MI355X.

The compute lives in a C-ABI HIP library (csrc/, declared in include/moe.h); `binding` marshals
torch tensors to it.  Importing the package does not load the library; `binding.lib()` does, and
fails loudly if it has not been built.
"""
