"""CPU oracle of the CoCoA round.  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's CPU-baseline leg may import this
package.  It imports nothing from the GPU library, and the GPU library never imports it.
"""
from . import policies  # noqa: F401
from .cocoa import OracleCoCoA, assign_greedy, build_oracle, projected_round_time  # noqa: F401
