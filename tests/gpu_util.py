"""The GPU tests take their device helpers (buffers through PyTorch, every computation through the C ABI) from the
harness module beside bench.py."""
from harness import *  # noqa: F401,F403
from harness import DEV, GpuModel  # noqa: F401
