"""CPU oracle for the phrase-boosting tree -- TEST INFRASTRUCTURE, NOT THE PRODUCT.

Only the tests, the smoke check and the benchmark's cpu_baseline leg may import
this package.  It shares no code with the HIP path and never imports it.
"""
from .pb_oracle import OracleTree, OracleError, build_library, oracle_threads, set_oracle_threads  # noqa: F401
