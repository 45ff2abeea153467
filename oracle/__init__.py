"""CPU oracle of the cascading KV cache.  Test infrastructure only.

Only the tests, the smoke check and the CPU-baseline leg of the benchmark may
import this package; the product (the HIP library and its binding) never does.
"""
from .cascade_oracle import OracleConfig, OracleSeq, build_oracle, oracle_library_path  # noqa: F401
