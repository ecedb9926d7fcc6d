"""CPU oracle for the I-ViT integer-only encoder forward.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package; the product path never does.  See ivit_oracle.c for the arithmetic.
"""
from .oracle import *  # noqa: F401,F403
