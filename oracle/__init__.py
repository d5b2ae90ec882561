"""CPU oracle of the lognormal gradient-compression path -- TEST INFRASTRUCTURE ONLY.

Only `tests/`, `__graft_entry__.smoke()` and the `cpu_baseline` leg of `bench.py` may import
this package.  The product (the HIP library and its Python binding) never does.
"""
from .lgn_oracle import *  # noqa: F401,F403
