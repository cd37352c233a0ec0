"""MI355X-native MoE expert-layer hot path: thin Python binding over libmoe_hip.so.

Importing the package loads nothing; `paper_2603_07685_amd.binding` loads the HIP
library on first use and fails loudly if it has not been built.
"""
__all__ = ["workloads"]
