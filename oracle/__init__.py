"""CPU oracle for GNND / GGM: test infrastructure, never part of the product path.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg import this
package.  It shares no code with the HIP implementation.
"""
from .gnnd_oracle import *  # noqa: F401,F403
