"""MI355X-native MBConv training step (forward + backward) behind a C ABI.

``binding`` mirrors include/mbconv.h; ``harness`` holds device buffers (PyTorch-ROCm
tensors, used for memory and the stream only) for tests and the benchmark.
"""
from . import binding  # noqa: F401
