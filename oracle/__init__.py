"""CPU oracle for the compressed-shard hot path (test infrastructure, not product code).

Plain, slow, single-purpose numpy implementations of the two compression techniques of the
paper's section "Compression techniques":

* item 1, dynamic blockwise quantization of the hidden states exchanged between nodes
  (``oracle.dynamic_code`` and ``oracle.blockwise_codec``);
* item 2, mixed matrix decomposition: int8 weights and activations with a small fp16 part for
  the critical (outlier) feature dimensions (``oracle.mixed_linear``).

Nothing in here is imported by the GPU library or its Python binding, and nothing in here
imports them.  Only tests, the smoke check and the CPU-baseline leg of the benchmark may use
this package.  Every function follows the step order of the method's definition with no
blocking, fusion or reordering, so that it can be checked against the definition by eye.
"""
