"""The GPU parity tests use the package's host<->device plumbing."""
from paper_2505_19201_amd.harness import *  # noqa: F401,F403
from paper_2505_19201_amd.harness import DT, TORCH_DT  # noqa: F401
