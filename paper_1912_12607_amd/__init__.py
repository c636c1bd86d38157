"""MI355X-native INT8 training convolution path (per-tensor INT8 quantizers, the
Direction Sensitive Gradient Clipping search, and int8 forward / backward-data /
backward-weight convolutions) behind a small C-ABI library.

Sub-modules are imported on demand: ``inputs`` (seeded synthetic tensors, no
arithmetic of the method) must stay importable without the HIP library, while
``binding`` loads ``csrc/libint8t.so`` and fails loudly when it is missing.
"""
__all__ = ["inputs", "binding"]
