"""CPU oracle for GVote's budget-free KV-cache selection path.

TEST INFRASTRUCTURE ONLY.  This package is the slow, plain, fp64 statement of
what the method computes, written from the paper (Sec. 3.1, Sec. 3.2 Steps 2-4,
Algorithm 1, Eq. (1), Sec. 3.4).  Only tests, the smoke check and the
benchmark's cpu_baseline leg may import it; the product path never does, and it
imports nothing from the HIP package.

Pin status of each function is stated in `oracle/gvote_oracle.py`'s header.
"""
from .gvote_oracle import *  # noqa: F401,F403
