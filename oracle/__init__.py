"""CPU oracle (test infrastructure only).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
package.  It shares no code with the HIP decoder.
"""
from .wfst_oracle import (Oracle, OracleResult, build_oracle, oracle_cutoff, oracle_keep,
                          ORACLE_LIB)

__all__ = ["Oracle", "OracleResult", "build_oracle", "oracle_cutoff", "oracle_keep", "ORACLE_LIB"]
