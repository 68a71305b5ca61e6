"""Shared test plumbing, kept under one name for the test files: host workload -> device tensors
(workloads/device.py) and the two comparers of the parity bar (oracle/compare.py: attention max-abs
error; acceptance with near-tie accounting)."""
from oracle.compare import NEAR_TIE, compare_accept, compare_accept_tree, compare_attention  # noqa: F401
from workloads.device import _torch_from, to_device  # noqa: F401
