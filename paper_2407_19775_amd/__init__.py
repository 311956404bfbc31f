"""MI355X-native mixed int8 linear layer and dynamic blockwise 8-bit codec.

The compute lives in a HIP shared library with a C ABI (see ``include/mmd8.h``); ``binding``
marshals torch device tensors into it.  Importing the package does not load the library; the
first call through ``binding`` does, and fails loudly if it has not been built.
"""
__all__ = ["binding", "workloads", "build"]
