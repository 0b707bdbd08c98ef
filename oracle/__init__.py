"""CPU oracle for the token-routed any-precision linear layer (test infrastructure).

Only the tests, the smoke check and the bench's CPU-baseline leg may import this
package.  It shares no code with the HIP library and never calls it.
"""
from .mbq_oracle import *  # noqa: F401,F403
