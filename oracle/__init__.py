"""fp64 CPU oracle for gist-masked causal attention.

TEST INFRASTRUCTURE ONLY: nothing in the product package may import this.
It shares no code with the HIP path.
"""
from .unigist_oracle import *  # noqa: F401,F403
from .fp8_e4m3 import *  # noqa: F401,F403,E402
