"""CPU oracle — TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg import this
package.  It never imports the product package and shares no code with it.
"""
from .oracle import Oracle, ORC_BF16, ORC_E4M3, OracleError  # noqa: F401
