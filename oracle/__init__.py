"""CPU oracle for the paged multi-LoRA delta (test infrastructure, not the product).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
package.  It loads oracle/liboracle.so (built from plora_oracle.cpp by build()) through
ctypes and shares nothing with the HIP library.
"""
from .pool import OraclePool, build, OracleError  # noqa: F401
from .manager import OracleManager  # noqa: F401
