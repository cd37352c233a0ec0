"""CPU oracle for the MoE expert-layer path: TEST INFRASTRUCTURE ONLY.

Thin numpy/ctypes front end of `moe_oracle.c` and `fp8_oracle.c` plus the
composition of the steps into a layer forward / backward in the order the paper
gives them (Sec. 2.1.1: route, dispatch(permute), compute, combine).  Nothing in
the product package imports this; it imports nothing from the product package.
"""
from .moe_oracle import *  # noqa: F401,F403
