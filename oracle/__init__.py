"""CPU oracle for SGD matrix factorization: test infrastructure only.

Nothing in the product package imports this; only tests, the smoke check and the
benchmark's cpu_baseline leg do.
"""
from .mf_oracle import *  # noqa: F401,F403
