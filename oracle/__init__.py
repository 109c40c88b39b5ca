"""CPU oracle for the pruned-prefill hot path.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package may import this
package; it is used by the tests, by the smoke check and by the benchmark's
CPU-baseline leg.  It shares no code with the HIP path.
"""
from .mvla_oracle import *  # noqa: F401,F403
